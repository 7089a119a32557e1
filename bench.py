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
        ("up_fwd", 0, 0, M, Il, H), ("down_fwd", 0, 0, M, H, Il),          # the MLP chain is enqueued first
        ("qkv_fwd", 0, 0, M, 3 * Hl, H), ("out_fwd", 0, 0, M, H, Hl),
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
    return ({
        "metric": "GB/s of algorithmic HBM bytes, replicated LayerNorm fwd+bwd", "value": round(gbs, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"LayerNorm on [M={M}, H={H}] of config {cfg.cfg_id}: {cfg.name}"},
        "roofline": {"kernel": "ln_fwd_kernel + ln_bwd_fused_kernel", "bound": "hbm",
                     "achieved": round(gbs, 1), "peak": 8000.0, "unit": "GB/s", "frac": round(gbs / 8000.0, 4),
                     "traffic": None, "fwd": {"ms": round(fwd_ms, 4), "GBps": round(fwd_bytes / fwd_ms / 1e6, 1)},
                     "bwd": {"ms": round(bwd_ms, 4), "GBps": round(bwd_bytes / bwd_ms / 1e6, 1)}},
        "cpu_baseline": {"value": round((fwd_bytes + bwd_bytes) / cpu_s / 1e9, 2), "unit": "GB/s", "cores": os.cpu_count(),
                         "kind": "oracle", "sample": "full workload, one fwd+bwd pass", "seconds": round(cpu_s, 2)},
        "max_rel_err_vs_oracle": err})


def bench_memopt(args, cfg, dt, pkg, torch, synthetic):
    """One rank's local compute in the memory-optimised distribution at the config's widths: every phase
    between collectives, forward and backward.  What the collectives would deliver (all-reduced moments,
    reduce-scattered slices, all-gathered gradients) is stood in for by fixed seeded tensors prepared before
    the timed region, so the time is the rank's kernels only."""
    import numpy as np
    from paper_2111_05972_amd.memopt import MemOptRank, PARAM_SHAPES
    from oracle import memopt_oracle as mo
    from oracle import max_rel_err
    H, nh, T, S, Bz = cfg.hidden, cfg.heads, cfg.tp_degree, cfg.seq, cfg.micro_batch
    I = cfg.intermediate or 4 * H
    rank = MemOptRank(H, nh, I, T, S, Bz, dt, cfg.causal, 1e-5)
    M, Hs, Hl, Il = rank.M, rank.Hs, rank.Hl, rank.Il
    sw = cfg.sigma_w if hasattr(cfg, "sigma_w") else 0.02

    def draw(seed, shape, sigma, mean=0.0):
        v = synthetic.normal(9000 + seed, int(np.prod(shape)), sigma) + np.float32(mean)
        return synthetic.quantize(v, cfg.dtype).reshape(shape)
    t0 = time.time()
    hp = {k: draw(i, sh, sw if k[0] in "wb" and k not in ("b1", "b2") else 0.1, 1.0 if k in ("g1", "g2") else 0.0)
          for i, (k, sh) in enumerate(PARAM_SHAPES(H, Hs, Hl, I, Il).items())}
    hin = {"x": draw(20, (M, Hs), 1.0), "qkv_in": draw(21, (M, 3 * Hl), 1.0), "o_in": draw(22, (M, Hs), 1.0),
           "u_in": draw(23, (M, Il), 1.0), "d_in": draw(24, (M, Hs), 1.0), "dy2": draw(25, (M, Hs), 1.0),
           "dy2_full": draw(26, (M, H), 1.0), "du_full": draw(27, (M, I), 1.0), "dy1_full": draw(28, (M, H), 1.0),
           "dqkv_full": draw(29, (M, 3 * H), 1.0)}
    # all-reduced moments / sums: T times a plausible local share (unit-variance channels)
    htot = {"m1": np.stack([np.zeros(M), np.full(M, float(H))], 1).astype(np.float32),
            "m2": np.stack([np.zeros(M), np.full(M, 2.0 * H)], 1).astype(np.float32),
            "s2": draw(30, (M, 2), 10.0).astype(np.float32), "s1": draw(31, (M, 2), 10.0).astype(np.float32)}
    p = {k: pkg.to_device(v, dt) for k, v in hp.items()}
    x = {k: pkg.to_device(v, dt) for k, v in hin.items()}
    tot = {k: torch.from_numpy(v).cuda() for k, v in htot.items()}
    gen_s = time.time() - t0
    stream = torch.cuda.current_stream()

    def step():
        rank.f0_moments(p, x["x"]); rank.f1_qkv_partial(tot["m1"]); rank.f2_attn_partial(x["qkv_in"])
        rank.f3_moments(x["o_in"]); rank.f4_up_partial(tot["m2"]); rank.f5_down_partial(x["u_in"])
        rank.f6_finish(x["d_in"])
        rank.b0_start(x["dy2"]); rank.b1_down(x["dy2_full"]); rank.b2_up(x["du_full"]); rank.b3_ln2(tot["s2"])
        rank.b4_attn(x["dy1_full"]); rank.b5_qkv(x["dqkv_full"]); rank.b6_ln1(tot["s1"])
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = 1e3 * (time.perf_counter() - t1) / args.steps
    f_fwd, f_bwd = cfg.flops()          # the same model flops as the speed-optimised shard: only the split axis differs
    tflops = (f_fwd + f_bwd) / (ms * 1e-3) / 1e12
    roofline = None
    if not args.no_kernel_timing:
        gl = [("qkv_fwd", M, 3 * H, Hs), ("out_fwd", M, H, Hl), ("up_fwd", M, I, Hs), ("down_fwd", M, H, Il),
              ("down_dgrad", M, Il, H), ("down_wgrad", Il, H, M), ("up_dgrad", M, Hs, I), ("up_wgrad", Hs, I, M),
              ("out_dgrad", M, Hl, H), ("out_wgrad", Hl, H, M), ("qkv_dgrad", M, Hs, 3 * H), ("qkv_wgrad", Hs, 3 * H, M)]
        reps = max(3, min(args.steps, 10))
        pkg.tp_layer_profile(1)
        for _ in range(reps):
            step()
        torch.cuda.synchronize()
        tms = pkg.tp_layer_profile_read()
        pkg.tp_layer_profile(0)
        assert len(tms) == 12 * reps, len(tms)
        per = [sum(tms[i::12]) / reps for i in range(12)]
        fl = [2.0 * g[1] * g[2] * g[3] for g in gl]
        ach = sum(fl) / (sum(per) * 1e-3) / 1e12
        roofline = {"kernel": "gemm_bf16 kernels (12 launches per step)", "bound": "mfma", "achieved": round(ach, 2),
                    "peak": BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(ach / BF16_PEAK_TFLOPS, 4), "traffic": None,
                    "gemm_ms_per_step": round(sum(per), 4),
                    "launches": {g[0]: {"M": g[1], "N": g[2], "K": g[3], "ms": round(t, 4),
                                        "tflops": round(f / t / 1e9, 1)} for g, t, f in zip(gl, per, fl)}}
    cpu_baseline, err = None, None
    if not args.no_cpu_baseline:
        step()
        torch.cuda.synchronize()
        N = lambda t: t.float().cpu().numpy()   # noqa: E731
        c0 = time.perf_counter()
        mean1, rstd1 = mo.ln_stats(htot["m1"], H, 1e-5)
        h1 = mo.ln_apply_fwd(hin["x"], mean1, rstd1, hp["g1"], hp["b1"])
        part_qkv = mo.linear_part_fwd(h1, hp["w_qkv"])
        y1 = mo.slice_epilogue_fwd(hin["o_in"], hp["b_o"], hin["x"])[1]
        mean2, rstd2 = mo.ln_stats(htot["m2"], H, 1e-5)
        h2 = mo.ln_apply_fwd(y1, mean2, rstd2, hp["g2"], hp["b2"])
        part_up = mo.linear_part_fwd(h2, hp["w_up"])
        u, g = mo.slice_epilogue_fwd(hin["u_in"], hp["b_up"], None, "gelu")
        part_dn = mo.linear_part_fwd(g, hp["w_dn"])
        y2 = mo.slice_epilogue_fwd(hin["d_in"], hp["b_dn"], y1)[1]
        dg, dw_dn = mo.linear_part_bwd(g, hp["w_dn"], hin["dy2_full"])
        du, db_up = mo.slice_epilogue_bwd(dg, u, "gelu")
        dh2, dw_up = mo.linear_part_bwd(h2, hp["w_up"], hin["du_full"])
        dy1, dg2, db2 = mo.ln_apply_bwd(dh2, y1, mean2, rstd2, hp["g2"], htot["s2"], H)
        dy1 = dy1 + hin["dy2"]
        dh1, dw_qkv = mo.linear_part_bwd(h1, hp["w_qkv"], hin["dqkv_full"])
        dx, dg1, db1 = mo.ln_apply_bwd(dh1, hin["x"], mean1, rstd1, hp["g1"], htot["s1"], H)
        cpu_s = time.perf_counter() - c0
        # the oracle pass above leaves out attention and the out-projection pair (3 of the 12 GEMMs)
        done = f_fwd + f_bwd - 3 * 2.0 * M * H * Hl - 3 * 4.0 * Bz * (nh // T) * (S * (S + 1) / 2 if cfg.causal else S * S) * (H // nh)
        try:
            from threadpoolctl import threadpool_info
            cores = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count()
        cpu_baseline = {"value": round(done / cpu_s / 1e12, 4), "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
                        "sample": "this rank's LayerNorm pieces, slice epilogues and 9 of its 12 GEMMs at full size, one pass",
                        "seconds": round(cpu_s, 2)}
        # backward of the last forward phase ran on u from the library's own (rounded) forward: compare what does not depend on it
        got = {"y2": (rank.y2, y2), "dx": (rank.dx, dx + dy1), "w_dn": (rank.grads["w_dn"], dw_dn),
               "w_up": (rank.grads["w_up"], dw_up), "w_qkv": (rank.grads["w_qkv"], dw_qkv), "b_up": (rank.grads["b_up"], db_up),
               "g2": (rank.grads["g2"], dg2), "g1": (rank.grads["g1"], dg1), "part_dn": (rank._part(H), part_dn)}
        err = max(max_rel_err(N(a), b) for a, b in got.values())
    return ({
        "metric": "TFLOP/s (fwd+bwd), one rank's local compute, memory-optimised distribution; % bf16 MFMA peak",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic", "pct_of_peak": round(100.0 * tflops / BF16_PEAK_TFLOPS, 2),
        "config": {"workload": f"memory-optimised local compute at the widths of config {cfg.cfg_id}: {cfg.name}",
                   "hidden": H, "heads": nh, "tp_degree": T, "seq": S, "micro_batch": Bz, "causal": cfg.causal,
                   "model_tflop_per_step": round((f_fwd + f_bwd) / 1e12, 4),
                   "collectives": "stood in for by fixed seeded tensors; not timed"},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "max_rel_err_vs_oracle": err, "input_gen_s": round(gen_s, 1)})


def _cores():
    try:
        from threadpoolctl import threadpool_info
        return int(max([i.get("num_threads", 1) for i in threadpool_info()] or [1]))
    except Exception:
        return os.cpu_count()


def _rms_rel(got, ref):
    import numpy as np
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    den = np.sqrt(np.mean(ref * ref))
    return float(np.sqrt(np.mean((got - ref) ** 2)) / den) if den > 0 else 0.0


def bench_layer(args, cfg, dt, pkg, torch, synthetic, ckpt=False, extras=True, oracle_limit=3.0e12, graph=False):
    """tp_layer_fwd + tp_layer_bwd (or tp_layer_bwd_recompute) on one config; returns the result as a dict.

    extras: also time the plain single-stream schedule, the row-epilogue variant and each GEMM launch (headline run).
    oracle_limit: the oracle runs on the full workload when its model flops are below this, else on a quarter of
    the tokens (timing only, no error figure).  graph: also capture fwd + bwd into a HIP graph and time replays."""
    peak = F32_PEAK_TFLOPS if cfg.dtype == "f32" else BF16_PEAK_TFLOPS
    t0 = time.time()
    d = synthetic.make_inputs(cfg)
    host_sh = pkg.shard_params(d, cfg.tp_degree if cfg.global_params else 1,
                               cfg.tp_rank if cfg.global_params else 0)
    mk_layer = lambda side, epi=cfg.row_epilogue: pkg.TpLayer(  # noqa: E731
        cfg.hidden, cfg.heads, cfg.tp_degree, cfg.tp_rank, cfg.seq, cfg.micro_batch, dt, cfg.causal, epi,
        cfg.head_dim, cfg.intermediate, side_stream=side)
    layer = mk_layer(not args.single_stream)
    p = {k: pkg.to_device(v, dt) for k, v in host_sh.items()}
    x = {k: pkg.to_device(d[k], dt) for k in ("x_a", "x_m", "dy_a", "dy_m")}
    y_a, y_m = layer.empty_outputs()
    dx_a, dx_m = layer.empty_outputs()
    grads = layer.empty_grads()
    stream = torch.cuda.current_stream()
    gen_s = time.time() - t0
    ws_ckpt = torch.empty(pkg.tp_layer_workspace_bytes_recompute(layer.desc), dtype=torch.uint8,
                          device="cuda") if ckpt else None

    def make_step(lay, g=grads):
        def step():
            lay.forward(p, x["x_a"], x["x_m"], y_a, y_m, stream=stream)
            if ckpt:    # backward recomputes QKV, O, LSE, U, G from the block inputs instead of reading `saved`
                pkg.tp_layer_bwd_recompute(lay.desc, p, x["x_a"], x["x_m"], x["dy_a"], x["dy_m"], g, dx_a, dx_m,
                                           ws_ckpt, stream=stream)
            else:
                lay.backward(p, x["x_a"], x["x_m"], x["dy_a"], x["dy_m"], g, dx_a, dx_m, stream=stream)
        return step
    step = make_step(layer)

    def timed(fn, n):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(n):
            fn()
        e1.record(stream)
        e1.synchronize()
        return e0.elapsed_time(e1) / n

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = 1e3 * (time.perf_counter() - t1) / args.steps
    f_fwd, f_bwd = cfg.flops()
    tflops = (f_fwd + f_bwd) / (ms_per_step * 1e-3) / 1e12
    n_split = max(3, min(args.steps, 10))
    fwd_ms = timed(lambda: layer.forward(p, x["x_a"], x["x_m"], y_a, y_m, stream=stream), n_split)
    out = {
        "metric": "TFLOP/s (fwd+bwd) per TP-rank layer shard on 1 MI355X; % bf16 MFMA peak",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "pct_of_peak": round(100.0 * tflops / peak, 2), "peak_tflops": peak,
        "fwd_ms": round(fwd_ms, 4), "bwd_ms": round(ms_per_step - fwd_ms, 4),
        "config": {"workload": f"config {cfg.cfg_id}: {cfg.name}" + (" (activation-checkpoint backward)" if ckpt else ""),
                   "hidden": cfg.hidden, "heads": cfg.heads, "head_dim": cfg.head_dim, "tp_degree": cfg.tp_degree,
                   "tp_rank": cfg.tp_rank, "seq": cfg.seq, "micro_batch": cfg.micro_batch, "causal": cfg.causal,
                   "row_epilogue": cfg.row_epilogue, "model_tflop_per_step": round((f_fwd + f_bwd) / 1e12, 4),
                   "schedule": "one stream" if args.single_stream else "two chains (TPL_SIDE_STREAM)",
                   "params": "shard generated directly" if not cfg.global_params else "sliced from unsharded"},
    }

    # A/B of the schedule: the same step with every kernel on the caller's stream
    if extras and not args.single_stream:
        lay1 = mk_layer(False)
        s1 = make_step(lay1)
        s1(); s1()
        one_ms = timed(s1, n_split)
        out["single_stream"] = {"ms_per_step": round(one_ms, 4), "value": round((f_fwd + f_bwd) / (one_ms * 1e-3) / 1e12, 2),
                                "steps": n_split, "what": "the same step without TPL_SIDE_STREAM (every kernel on the caller's stream)"}
        del lay1
    # the same shard with the row-parallel epilogue on (bias + residual in the two row-parallel GEMMs, residual
    # gradients in the two input-gradient GEMMs, db_o and db_dn): the headline rank runs with it off
    if extras and not cfg.row_epilogue and not ckpt and not args.no_row_epilogue_variant:
        layer_on = mk_layer(not args.single_stream, True)
        grads_on = layer_on.empty_grads()
        step_on = make_step(layer_on, grads_on)
        step_on(); step_on()
        on_ms = timed(step_on, n_split)
        out["row_epilogue_on"] = {"ms_per_step": round(on_ms, 4), "value": round((f_fwd + f_bwd) / (on_ms * 1e-3) / 1e12, 2),
                                  "steps": n_split, "what": "same shard with the bias + residual epilogue of the row-parallel GEMMs on"}
        del layer_on, grads_on

    # dominant kernel: the GEMM kernel.  Its 12 launches per step are timed inside real steps: the
    # library brackets each GEMM launch with HIP events on the launch stream (tp_layer_profile).
    roofline = None
    if not args.no_kernel_timing:
        names = [g_[0] for g_ in gemm_list(cfg)]
        flops = {g_[0]: 2.0 * g_[3] * g_[4] * g_[5] for g_ in gemm_list(cfg)}
        shapes = {g_[0]: {"M": g_[3], "N": g_[4], "K": g_[5]} for g_ in gemm_list(cfg)}
        reps = max(3, min(args.steps, 10))
        pkg.tp_layer_profile(1)
        for _ in range(reps):
            step()
        torch.cuda.synchronize()
        ms = pkg.tp_layer_profile_read()
        pkg.tp_layer_profile(0)
        per_step = len(ms) // reps          # 12, or 14 with the recomputed QKV and up-projection GEMMs
        assert len(ms) == per_step * reps and per_step in (12, 14), len(ms)
        if per_step == 14:                  # launch order: 4 fwd, then recomputed up_fwd and qkv_fwd, then 8 bwd
            order = names[:4] + ["up_fwd", "qkv_fwd"] + names[4:]
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
        roofline = {"kernel": "bf16 MFMA GEMM kernels of gemm_bf16.hip (12 launches per step, one at a time)" if cfg.dtype == "bf16" else "gemm_simple_kernel",
                    "bound": "mfma" if cfg.dtype == "bf16" else "alu",
                    "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s",
                    "frac": round(achieved / peak, 4), "traffic": traffic,
                    "flops_per_launch": tot_fl / 12, "avg_launch_ms": round(tot_ms / 12, 4),
                    "gemm_ms_per_step": round(tot_ms, 4)}
        if extras:
            roofline["launches"] = {n: {**shapes[n], "ms": round(per[n], 4), "tflops": round(flops[n] / per[n] / 1e9, 1)} for n in names}
    out["roofline"] = roofline

    cpu_baseline, max_err, rms_err = None, None, None
    if not args.no_cpu_baseline:
        import oracle
        from synthetic.configs import small_variant
        scfg, sample = cfg, "full workload, one fwd+bwd pass"
        if sum(cfg.flops()) > oracle_limit:
            scfg = small_variant(cfg, seq=max(1, cfg.seq // 4))
            sample = f"same widths, seq {scfg.seq} (1/4 of the tokens), one fwd+bwd pass"
        sd = d if scfg is cfg else {k: (v[:scfg.tokens] if k in ("x_a", "x_m", "dy_a", "dy_m") else v) for k, v in d.items()}
        # the oracle shards with its own rule (the product sharded the GPU side above)
        osh = oracle.shard_params(d, cfg.tp_degree if cfg.global_params else 1, cfg.tp_rank if cfg.global_params else 0)
        a = (scfg.micro_batch, scfg.seq, scfg.local_heads, scfg.head_dim, scfg.causal, scfg.row_epilogue)
        c0 = time.perf_counter()
        ya, ym, osv = oracle.layer_fwd(sd["x_a"], sd["x_m"], osh, *a)
        ref = oracle.layer_bwd(sd["x_a"], sd["x_m"], osh, sd["dy_a"], sd["dy_m"], osv, *a)
        cpu_s = time.perf_counter() - c0
        cpu_baseline = {"value": round(sum(scfg.flops()) / cpu_s / 1e12, 4), "unit": "TFLOP/s", "cores": _cores(),
                        "kind": "oracle", "sample": sample, "seconds": round(cpu_s, 2)}
        if scfg is cfg:
            ref.update(y_a=ya, y_m=ym)
            got = {"y_a": y_a, "y_m": y_m, "dx_a": dx_a, "dx_m": dx_m, **grads}
            step()
            torch.cuda.synchronize()
            host = {k: v.float().cpu().numpy() for k, v in got.items() if k in ref}
            max_err = max(oracle.max_rel_err(v, ref[k]) for k, v in host.items())
            rms_err = max(_rms_rel(v, ref[k]) for k, v in host.items())
    out.update(cpu_baseline=cpu_baseline, max_rel_err_vs_oracle=max_err, rms_rel_err_vs_oracle=rms_err,
               input_gen_s=round(gen_s, 1))
    # the step captured by the caller into a HIP graph and replayed (launch-bound shapes)
    if graph and not ckpt:
        try:
            side = torch.cuda.Stream()
            g = torch.cuda.CUDAGraph()
            side.wait_stream(stream)
            with torch.cuda.stream(side):
                cap_stream = torch.cuda.current_stream()

                def cap_step():
                    layer.forward(p, x["x_a"], x["x_m"], y_a, y_m, stream=cap_stream)
                    layer.backward(p, x["x_a"], x["x_m"], x["dy_a"], x["dy_m"], grads, dx_a, dx_m, stream=cap_stream)
                cap_step()
                torch.cuda.synchronize()
                with torch.cuda.graph(g, stream=side):
                    cap_step()
            stream.wait_stream(side)
            for _ in range(3):
                g.replay()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(args.steps):
                g.replay()
            torch.cuda.synchronize()
            gms = 1e3 * (time.perf_counter() - t1) / args.steps
            out["graph_replay"] = {"ms_per_step": round(gms, 4), "value": round((f_fwd + f_bwd) / (gms * 1e-3) / 1e12, 2),
                                   "what": "tp_layer_fwd + tp_layer_bwd captured by the caller into one HIP graph, replayed"}
        except Exception as e:      # capture is the caller's business; the eager figure stands
            out["graph_replay"] = {"error": str(e)[:200]}

    return out


def bench_layer_ln(args, cfg, dt, pkg, torch, synthetic):
    """One rank's kernels for a whole post-LN layer pass (Sec. I.1 / I.4): the shard forward, LN1 on the attention
    block's sum and LN2 on the MLP block's sum; backward through LN2, the shard and LN1.  The all-reduces are not run
    (one GPU): where the group's sum is needed the rank's own partial stands in, and the MLP block's input is the LN1
    output of the previous pass, so every pass runs exactly the kernels a rank runs per layer.  Values are checked by
    tests/test_gpu_ln_compose.py (all ranks on one GPU, against the oracle); this is timing only."""
    M, H = cfg.tokens, cfg.hidden
    tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    d = synthetic.make_inputs(cfg)
    host_sh = pkg.shard_params(d, cfg.tp_degree if cfg.global_params else 1, cfg.tp_rank if cfg.global_params else 0)
    layer = pkg.TpLayer(cfg.hidden, cfg.heads, cfg.tp_degree, cfg.tp_rank, cfg.seq, cfg.micro_batch, dt, cfg.causal,
                        cfg.row_epilogue, cfg.head_dim, cfg.intermediate, side_stream=not args.single_stream)
    p = {k: pkg.to_device(v, dt) for k, v in host_sh.items()}
    x = {k: pkg.to_device(d[k], dt) for k in ("x_a", "x_m", "dy_a", "dy_m")}
    st = torch.cuda.current_stream()
    y_a, y_m = layer.empty_outputs()
    dx_a, dx_m = layer.empty_outputs()
    grads = layer.empty_grads()
    gam = [torch.ones(H, dtype=tdt, device="cuda") for _ in range(2)]
    bet = [torch.zeros(H, dtype=tdt, device="cuda") for _ in range(2)]
    x_m, out, d_ya, d_ym = (torch.empty(M, H, dtype=tdt, device="cuda") for _ in range(4))
    x_m.copy_(x["x_m"]); d_ya.copy_(x["dy_a"])
    mean = [torch.empty(M, dtype=torch.float32, device="cuda") for _ in range(2)]
    rstd = [torch.empty(M, dtype=torch.float32, device="cuda") for _ in range(2)]
    dg, db = torch.empty_like(gam[0]), torch.empty_like(gam[0])
    ws = torch.empty(pkg.tp_layer_ln_workspace_bytes(M, H), dtype=torch.uint8, device="cuda")

    def fwd():
        layer.forward(p, x["x_a"], x_m, y_a, y_m, stream=st)
        pkg.tp_layer_ln_fwd(dt, M, H, y_a, None, gam[0], bet[0], 1e-5, None, x_m, mean[0], rstd[0], stream=st)
        pkg.tp_layer_ln_fwd(dt, M, H, y_m, None, gam[1], bet[1], 1e-5, None, out, mean[1], rstd[1], stream=st)

    def bwd():
        pkg.tp_layer_ln_bwd(dt, M, H, x["dy_m"], y_m, mean[1], rstd[1], gam[1], d_ym, dg, db, ws, stream=st)
        layer.backward(p, x["x_a"], x_m, d_ya, d_ym, grads, dx_a, dx_m, stream=st)
        pkg.tp_layer_ln_bwd(dt, M, H, dx_m, y_a, mean[0], rstd[0], gam[0], d_ya, dg, db, ws, stream=st)

    def timed(fn, n):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        for _ in range(n):
            fn()
        e1.record(st)
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
    fwd_ms = timed(fwd, max(3, min(args.steps, 10)))
    f_fwd, f_bwd = cfg.flops()
    peak = F32_PEAK_TFLOPS if cfg.dtype == "f32" else BF16_PEAK_TFLOPS
    tf = (f_fwd + f_bwd) / (ms * 1e-3) / 1e12
    assert torch.isfinite(out.float()).all() and torch.isfinite(d_ya.float()).all()
    return {"metric": "TFLOP/s (fwd+bwd) of one rank's kernels for a post-LN layer: shard + both LayerNorms; % of peak",
            "value": round(tf, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": cfg.dtype, "data": "synthetic", "pct_of_peak": round(100.0 * tf / peak, 2),
            "fwd_ms": round(fwd_ms, 4), "bwd_ms": round(ms - fwd_ms, 4),
            "config": {"workload": f"config {cfg.cfg_id}: {cfg.name} with its two LayerNorms (post-LN layer, one rank's kernels)"}}


def bench_attention(args, cfg, dt, pkg, torch, synthetic):
    """The attention kernels of the config alone (tp_layer_attn_fwd, tp_layer_attn_bwd on its [B, S, local heads, dh]),
    random inputs, no workspace (strips whole, as inside the layer): time and rate of each."""
    B, S, nl, dh, causal = cfg.micro_batch, cfg.seq, cfg.local_heads, cfg.head_dim, cfg.causal
    tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    st = torch.cuda.current_stream()
    qkv = torch.randn(B * S, 3 * nl * dh, device="cuda", dtype=tdt)
    o = torch.empty(B * S, nl * dh, device="cuda", dtype=tdt)
    d_o = torch.randn_like(o)
    lse = torch.empty(B, nl, S, device="cuda", dtype=torch.float32)
    dsum = torch.empty_like(lse)
    dqkv = torch.empty_like(qkv)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        for _ in range(args.steps):
            fn()
        e1.record(st)
        e1.synchronize()
        return e0.elapsed_time(e1) / args.steps
    fwd_ms = timed(lambda: pkg.tp_layer_attn_fwd(dt, B, S, nl, dh, causal, qkv, o, lse, stream=st))
    bwd_ms = timed(lambda: pkg.tp_layer_attn_bwd(dt, B, S, nl, dh, causal, qkv, o, lse, d_o, dqkv, dsum, stream=st))
    pairs = S * (S + 1) // 2 if causal else S * S
    flops = 4.0 * B * nl * pairs * dh
    peak = F32_PEAK_TFLOPS if cfg.dtype == "f32" else BF16_PEAK_TFLOPS
    tf = 3.0 * flops / ((fwd_ms + bwd_ms) * 1e-3) / 1e12
    return {"metric": "TFLOP/s of the attention kernels alone (forward + backward)", "value": round(tf, 1), "unit": "TFLOP/s",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(fwd_ms + bwd_ms, 4),
            "higher_is_better": True, "dtype": cfg.dtype, "data": "synthetic",
            "config": {"workload": f"attention of config {cfg.cfg_id}: {cfg.name} (B={B}, S={S}, local heads={nl}, dh={dh}, causal={causal})"},
            "fwd": {"ms": round(fwd_ms, 4), "tflops": round(flops / fwd_ms / 1e9, 1), "frac_of_peak": round(flops / fwd_ms / 1e9 / peak, 4)},
            "bwd": {"ms": round(bwd_ms, 4), "tflops": round(2 * flops / bwd_ms / 1e9, 1), "frac_of_peak": round(2 * flops / bwd_ms / 1e9 / peak, 4)}}


def bench_gemms(args, cfg, dt, pkg, torch, synthetic):
    """The 12 GEMMs of a step, each alone in a sustained loop on random operands: this library (tp_layer_gemm) and,
    as a reference point of what the chip sustains on the same shape, the vendor library behind torch.matmul.  Two
    regimes: `hot` (the same operands every launch: they stay in the 256 MB infinity cache) and `cold` (four operand
    sets in rotation, more than the cache holds, as inside a layer step where every weight is read once).  A host
    thread samples board power and core clock from sysfs during the hot loop (the GEMMs run at the power limit)."""
    import glob
    import threading
    st = torch.cuda.current_stream()
    hw = {}
    for h in glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*"):
        if os.path.exists(os.path.join(h, "power1_input")):
            hw.setdefault("power", os.path.join(h, "power1_input"))
    for q in glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"):
        hw.setdefault("sclk", q)

    def sample(stop, acc):
        while not stop.is_set():
            try:
                if "power" in hw:
                    acc["w"].append(float(open(hw["power"]).read()) / 1e6)
                if "sclk" in hw:
                    cur = [l for l in open(hw["sclk"]).read().splitlines() if "*" in l]
                    if cur:
                        acc["mhz"].append(float(cur[0].split(":")[1].lower().replace("mhz", "").replace("*", "").strip()))
            except Exception:
                pass
            time.sleep(0.05)

    def loop(fn, secs, sampled):
        for i in range(6):
            fn(i)
        torch.cuda.synchronize()
        stop, acc = threading.Event(), {"w": [], "mhz": []}
        th = threading.Thread(target=sample, args=(stop, acc)) if sampled else None
        if th:
            th.start()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0, n = time.time(), 0
        e0.record(st)
        while time.time() - t0 < secs:
            for i in range(40):
                fn(n + i)
            n += 40
            torch.cuda.synchronize()
        e1.record(st)
        e1.synchronize()
        stop.set()
        if th:
            th.join()
        half = lambda v: v[len(v) // 2:]   # noqa: E731
        avg = lambda v: round(sum(half(v)) / len(half(v)), 1) if v else None   # noqa: E731
        return e0.elapsed_time(e1) / n, avg(acc["w"]), avg(acc["mhz"])
    rows = {}
    secs = 0.6 if args.steps <= 30 else 1.5
    for name, ta, tb, M, N, K in gemm_list(cfg):
        nrot = 4
        As = [torch.randn((K, M) if ta else (M, K), device="cuda", dtype=torch.bfloat16) for _ in range(nrot)]
        Bs = [torch.randn((N, K) if tb else (K, N), device="cuda", dtype=torch.bfloat16) for _ in range(nrot)]
        C = torch.empty(M, N, device="cuda", dtype=torch.bfloat16)
        ws = torch.empty(max(256, pkg.tp_layer_gemm_workspace_bytes(dt, M, N, K)), dtype=torch.uint8, device="cuda")
        ours = lambda i, r: pkg.tp_layer_gemm(dt, ta, tb, M, N, K, As[i % r], Bs[i % r], C, ws=ws, stream=st)   # noqa: E731
        vend = lambda i, r: torch.matmul(As[i % r].t() if ta else As[i % r], Bs[i % r].t() if tb else Bs[i % r], out=C)   # noqa: E731
        fl = 2.0 * M * N * K
        row = {"M": M, "N": N, "K": K, "layout": ("T" if ta else "N") + ("T" if tb else "N")}
        for who, f in (("ours", ours), ("vendor", vend)):
            hot_ms, w, mhz = loop(lambda i: f(i, 1), secs, True)
            cold_ms, _, _ = loop(lambda i: f(i, nrot), secs, False)
            row[who] = {"hot_tflops": round(fl / hot_ms / 1e9, 1), "cold_tflops": round(fl / cold_ms / 1e9, 1),
                        "hot_watts": w, "hot_mhz": mhz}
        rows[name] = row
        del As, Bs, C
        torch.cuda.empty_cache()
    tot = lambda who, k: sum(2.0 * r["M"] * r["N"] * r["K"] for r in rows.values()) / sum(   # noqa: E731
        2.0 * r["M"] * r["N"] * r["K"] / r[who][k] for r in rows.values())
    return {"metric": "TFLOP/s of each GEMM of a step alone, sustained loop, random operands", "unit": "TFLOP/s",
            "value": round(tot("ours", "cold_tflops"), 1), "dtype": cfg.dtype, "data": "synthetic",
            "config": {"workload": f"the 12 GEMMs of config {cfg.cfg_id}: {cfg.name}, one at a time"},
            "flop_weighted": {who: {k: round(tot(who, k), 1) for k in ("hot_tflops", "cold_tflops")} for who in ("ours", "vendor")},
            "vendor": "torch.matmul (hipBLASLt / rocBLAS), a reference point only: not on the product path",
            "gemms": rows}


def _brief(r):
    """One workload's result cut down to what the `other_workloads` block carries."""
    keep = ("metric", "value", "unit", "ms_per_step", "dtype", "pct_of_peak", "fwd_ms", "bwd_ms", "max_rel_err_vs_oracle",
            "rms_rel_err_vs_oracle", "single_stream", "graph_replay")
    b = {k: r[k] for k in keep if k in r and r[k] is not None}
    b["workload"] = r["config"]["workload"]
    if r.get("roofline"):
        b["roofline"] = {k: r["roofline"][k] for k in ("bound", "achieved", "peak", "unit", "frac") if k in r["roofline"]}
    if r.get("cpu_baseline"):
        b["cpu_baseline"] = {k: r["cpu_baseline"][k] for k in ("value", "unit", "cores", "sample", "seconds") if k in r["cpu_baseline"]}
    return b


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="5")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true")
    ap.add_argument("--no-row-epilogue-variant", action="store_true",
                    help="skip the extra timing of the same shard with the row-parallel epilogue on")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="only the headline workload: skip the `other_workloads` block of the default run")
    ap.add_argument("--workload", default="layer", choices=["layer", "layer-checkpoint", "layer-ln", "ln", "memopt", "gemms", "attn"],
                    help="layer: tp_layer_fwd + tp_layer_bwd (the headline metric); layer-checkpoint: tp_layer_fwd + "
                         "tp_layer_bwd_recompute; ln: replicated LayerNorm forward + backward on the config's [M, H]; "
                         "memopt: one rank's local compute in the memory-optimised distribution at the config's widths; "
                         "gemms: each GEMM of a step alone in a sustained loop, beside the vendor library on the same shape, "
                         "with board power and clock; attn: the attention kernels of the config alone; layer-ln: the shard with the "
                         "two replicated LayerNorms of a post-LN layer around it, forward and backward")
    ap.add_argument("--single-stream", action="store_true",
                    help="time the plain schedule, every kernel on the caller's stream, instead of the two-chain "
                         "schedule (TPL_SIDE_STREAM: the MLP block of a pass on a second, library-owned stream)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device copy (reference point for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs one tensor-parallel rank's shard on ONE GPU; "
              "--gpus above 1 is not supported (no collectives in this path)", file=sys.stderr)
        sys.exit(2)

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
    if args.workload == "ln":
        print(json.dumps(bench_layernorm(args, cfg, dt, pkg, torch, synthetic)))
        return
    if args.workload == "memopt":
        print(json.dumps(bench_memopt(args, cfg, dt, pkg, torch, synthetic)))
        return
    if args.workload == "gemms":
        print(json.dumps(bench_gemms(args, cfg, dt, pkg, torch, synthetic)))
        return
    if args.workload == "attn":
        print(json.dumps(bench_attention(args, cfg, dt, pkg, torch, synthetic)))
        return
    if args.workload == "layer-ln":
        print(json.dumps(bench_layer_ln(args, cfg, dt, pkg, torch, synthetic)))
        return
    out = bench_layer(args, cfg, dt, pkg, torch, synthetic, ckpt=args.workload == "layer-checkpoint")

    # The default run also carries every other configuration and workload, each measured the same way (fewer steps;
    # the oracle on the full workload where that takes seconds), so that one line shows the whole picture.
    default_run = args.workload == "layer" and key == 5 and not args.no_other_workloads
    if default_run:
        import copy
        others = []
        oa = copy.copy(args)
        oa.steps, oa.warmup = max(5, min(args.steps, 20)), 3
        t_start = time.time()

        def attempt(what, fn):      # a failure here must not cost the headline line
            torch.cuda.empty_cache()
            try:
                others.append(_brief(fn()))
            except Exception as e:
                others.append({"workload": what, "error": str(e)[:300]})
        for k in (1, 2, 3, 4, "roberta-10b-tp4", "bert-10b-tp4"):
            c = synthetic.get_config(k)
            cdt = pkg.TPL_F32 if c.dtype == "f32" else pkg.TPL_BF16
            attempt(f"config {c.cfg_id}: {c.name}", lambda c=c, cdt=cdt, k=k: bench_layer(
                oa, c, cdt, pkg, torch, synthetic, extras=False,
                oracle_limit=2.5e12 if time.time() - t_start < 150 else 0.0, graph=k in (1, 2, 3)))
        attempt("layer-checkpoint", lambda: bench_layer(oa, cfg, dt, pkg, torch, synthetic, ckpt=True, extras=False,
                                                        oracle_limit=0.0))
        attempt("ln", lambda: bench_layernorm(oa, cfg, dt, pkg, torch, synthetic))
        attempt("layer-ln", lambda: bench_layer_ln(oa, cfg, dt, pkg, torch, synthetic))
        ma = copy.copy(oa)
        ma.no_cpu_baseline = args.no_cpu_baseline or time.time() - t_start > 200
        attempt("memopt", lambda: bench_memopt(ma, cfg, dt, pkg, torch, synthetic))
        out["other_workloads"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
