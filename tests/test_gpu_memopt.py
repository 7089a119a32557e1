"""GPU parity for the memory-optimised distribution's local compute (App. F.2 of the paper): each library
call against the oracle's definition, then T ranks simulated on the one GPU (the collectives emulated by
summing / slicing / concatenating their buffers) against the oracle's simulated ranks and its unsharded layer."""
import numpy as np
import pytest

import synthetic
from oracle import memopt_oracle as mo
from oracle import max_rel_err

pytestmark = pytest.mark.gpu

TOL = {"bf16": 2e-2, "f32": 1e-4}
# (M, Hs, T): ragged rows / partial column tile, several row slabs and column tiles, config 5's slice
SLICE_CASES = [(7, 40, 3), (300, 1048, 2), (33, 4096, 4), (2048, 1536, 8), (1, 8, 1)]


def _draw(seed, shape, sigma, dtype, mean=0.0):
    n = int(np.prod(shape))
    return synthetic.quantize(synthetic.normal(seed, n, sigma) + np.float32(mean), dtype).reshape(shape)


def _dt(pkg, dtype):
    return pkg.TPL_BF16 if dtype == "bf16" else pkg.TPL_F32


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_distributed_layernorm_pieces(dtype):
    import torch
    import paper_2111_05972_amd as pkg
    dt, tol, eps = _dt(pkg, dtype), TOL[dtype], 1e-5
    st = torch.cuda.current_stream()
    f32 = lambda *s: torch.empty(*s, dtype=torch.float32, device="cuda")   # noqa: E731
    for ci, (M, Hs, T) in enumerate(SLICE_CASES):
        H = Hs * T
        print(f"\n[memopt-ln] {dtype} M={M} Hs={Hs} H={H}", flush=True)
        x = _draw(1200 + ci, (M, Hs), 1.0, dtype, mean=0.3)
        gamma = _draw(1210 + ci, (Hs,), 0.2, dtype, mean=1.0)
        beta = _draw(1220 + ci, (Hs,), 0.2, dtype)
        dy = _draw(1230 + ci, (M, Hs), 1.0, dtype)
        dres = _draw(1240 + ci, (M, Hs), 1.0, dtype)
        # what the other T-1 ranks would contribute to the all-reduced moments and sums
        other_m = np.stack([np.full(M, 0.1 * (H - Hs)), np.full(M, 1.2 * (H - Hs))], axis=1).astype(np.float32)
        other_s = _draw(1250 + ci, (M, 2), 3.0, "f32") if T > 1 else np.zeros((M, 2), np.float32)
        D = lambda v: pkg.to_device(v, dt)   # noqa: E731
        x_d, g_d, b_d, dy_d, dres_d = D(x), D(gamma), D(beta), D(dy), D(dres)
        # 1. local moments
        sums_d = f32(M, 2)
        pkg.tp_layer_ln_moments(dt, M, Hs, x_d, sums_d, stream=st)
        ref_m = mo.ln_local_moments(x)
        assert max_rel_err(sums_d.cpu().numpy(), ref_m) <= tol
        # 2. statistics from the totals (the oracle's local moments + the other ranks' share)
        tot = (ref_m + other_m).astype(np.float32)
        tot_d = torch.from_numpy(tot).cuda()
        mean_d, rstd_d = f32(M), f32(M)
        pkg.tp_layer_ln_stats(M, H, eps, tot_d, mean_d, rstd_d, stream=st)
        mean_ref, rstd_ref = mo.ln_stats(tot, H, eps)
        assert max_rel_err(mean_d.cpu().numpy(), mean_ref) <= 1e-5
        assert max_rel_err(rstd_d.cpu().numpy(), rstd_ref) <= 1e-4
        # 3. ApplyLayerNorm
        y_d = torch.empty_like(x_d)
        pkg.tp_layer_ln_apply_fwd(dt, M, Hs, x_d, mean_d, rstd_d, g_d, b_d, y_d, stream=st)
        assert max_rel_err(y_d.float().cpu().numpy(), mo.ln_apply_fwd(x, mean_ref, rstd_ref, gamma, beta)) <= tol
        # 4. backward sums of the slice
        pkg.tp_layer_ln_apply_bwd_sums(dt, M, Hs, dy_d, x_d, mean_d, rstd_d, g_d, sums_d, stream=st)
        ref_s = mo.ln_apply_bwd_sums(dy, x, mean_ref, rstd_ref, gamma)
        assert max_rel_err(sums_d.cpu().numpy(), ref_s) <= tol
        # 5. backward apply with the totals, with and without a residual gradient
        tot_s = (ref_s + other_s).astype(np.float32)
        tot_s_d = torch.from_numpy(tot_s).cuda()
        ws = torch.empty(pkg.tp_layer_ln_apply_workspace_bytes(M, Hs), dtype=torch.uint8, device="cuda")
        dx_ref, dg_ref, db_ref = mo.ln_apply_bwd(dy, x, mean_ref, rstd_ref, gamma, tot_s, H)
        for add_d, ref in ((None, dx_ref), (dres_d, dx_ref + dres)):
            dx_d, dgam_d, dbet_d = torch.empty_like(x_d), torch.empty_like(g_d), torch.empty_like(g_d)
            pkg.tp_layer_ln_apply_bwd(dt, M, Hs, H, dy_d, x_d, mean_d, rstd_d, g_d, tot_s_d, add_d, dx_d, dgam_d,
                                      dbet_d, ws, stream=st)
            torch.cuda.synchronize()
            assert max_rel_err(dx_d.float().cpu().numpy(), ref) <= tol
            assert max_rel_err(dgam_d.float().cpu().numpy(), dg_ref) <= tol
            assert max_rel_err(dbet_d.float().cpu().numpy(), db_ref) <= tol


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_slice_epilogue(dtype):
    import torch
    import paper_2111_05972_amd as pkg
    dt, tol = _dt(pkg, dtype), TOL[dtype]
    st = torch.cuda.current_stream()
    for ci, (M, N) in enumerate([(7, 40), (300, 1048), (2048, 6144), (1, 8)]):
        print(f"\n[memopt-epilogue] {dtype} M={M} N={N}", flush=True)
        inp = _draw(1300 + ci, (M, N), 1.0, dtype)
        bias = _draw(1310 + ci, (N,), 0.5, dtype)
        res = _draw(1320 + ci, (M, N), 1.0, dtype)
        dout = _draw(1330 + ci, (M, N), 1.0, dtype)
        D = lambda v: pkg.to_device(v, dt)   # noqa: E731
        in_d, b_d, r_d, do_d = D(inp), D(bias), D(res), D(dout)
        ws = torch.empty(pkg.tp_layer_slice_epilogue_workspace_bytes(M, N), dtype=torch.uint8, device="cuda")
        # no activation, with and without residual
        for rd, rn in ((None, None), (r_d, res)):
            out_d = torch.empty_like(in_d)
            pkg.tp_layer_slice_epilogue_fwd(dt, pkg.TPL_ACT_NONE, M, N, in_d, b_d, rd, None, out_d, stream=st)
            assert max_rel_err(out_d.float().cpu().numpy(), mo.slice_epilogue_fwd(inp, bias, rn)[1]) <= tol
        db_d = torch.empty_like(b_d)
        pkg.tp_layer_slice_epilogue_bwd(dt, pkg.TPL_ACT_NONE, M, N, do_d, None, None, db_d, ws, stream=st)
        assert max_rel_err(db_d.float().cpu().numpy(), mo.slice_epilogue_bwd(dout)[1]) <= tol
        # bias + GeLU
        u_d, g_d = torch.empty_like(in_d), torch.empty_like(in_d)
        pkg.tp_layer_slice_epilogue_fwd(dt, pkg.TPL_ACT_GELU, M, N, in_d, b_d, None, u_d, g_d, stream=st)
        u_ref, g_ref = mo.slice_epilogue_fwd(inp, bias, None, "gelu")
        assert max_rel_err(u_d.float().cpu().numpy(), u_ref) <= tol
        assert max_rel_err(g_d.float().cpu().numpy(), g_ref) <= tol
        din_d = torch.empty_like(in_d)
        pkg.tp_layer_slice_epilogue_bwd(dt, pkg.TPL_ACT_GELU, M, N, do_d, u_d, din_d, db_d, ws, stream=st)
        torch.cuda.synchronize()
        u_stored = u_d.float().cpu().numpy()          # backward sees the stored (rounded) pre-activation
        din_ref, db_ref = mo.slice_epilogue_bwd(dout, u_stored, "gelu")
        assert max_rel_err(din_d.float().cpu().numpy(), din_ref) <= tol
        assert max_rel_err(db_d.float().cpu().numpy(), db_ref) <= tol


def _global_params(seed, H, nh, I, dtype):
    sw = 0.02
    g = {"nh": nh,
         "Wqkv": _draw(seed + 1, (H, 3 * H), sw, dtype), "bqkv": _draw(seed + 2, (3 * H,), sw, dtype),
         "Wo": _draw(seed + 3, (H, H), sw, dtype), "bo": _draw(seed + 4, (H,), sw, dtype),
         "Wup": _draw(seed + 5, (H, I), sw, dtype), "bup": _draw(seed + 6, (I,), sw, dtype),
         "Wdn": _draw(seed + 7, (I, H), sw, dtype), "bdn": _draw(seed + 8, (H,), sw, dtype),
         "g1": _draw(seed + 9, (H,), 0.1, dtype, mean=1.0), "b1": _draw(seed + 10, (H,), 0.1, dtype),
         "g2": _draw(seed + 11, (H,), 0.1, dtype, mean=1.0), "b2": _draw(seed + 12, (H,), 0.1, dtype)}
    return g


def _run_simulated_ranks(pkg, torch, dt, H, nh, I, T, S, Bz, causal, eps, shards, x, dy):
    """All T ranks on the one GPU, phase by phase; the collectives are emulated on their buffers."""
    from paper_2111_05972_amd.memopt import MemOptRank
    ranks = [MemOptRank(H, nh, I, T, S, Bz, dt, causal, eps) for _ in range(T)]
    Hs = H // T
    D = lambda v: pkg.to_device(v, dt)   # noqa: E731
    ps = [{k: D(v) for k, v in shards[r].items()} for r in range(T)]
    xs = [D(x[:, r * Hs:(r + 1) * Hs]) for r in range(T)]
    dys = [D(dy[:, r * Hs:(r + 1) * Hs]) for r in range(T)]

    def all_reduce(ts):
        tot = torch.stack([t.float() for t in ts]).sum(0)
        return [tot.clone() for _ in ts]

    def reduce_scatter(ts):
        tot = torch.stack([t.float() for t in ts]).sum(0)
        w = tot.shape[1] // T
        return [tot[:, r * w:(r + 1) * w].to(ts[0].dtype).contiguous() for r in range(T)]

    def all_gather(ts):
        full = torch.cat(ts, dim=1).contiguous()
        return [full for _ in ts]

    R = range(T)
    tot = all_reduce([ranks[r].f0_moments(ps[r], xs[r]) for r in R])
    q = reduce_scatter([ranks[r].f1_qkv_partial(tot[r]) for r in R])
    o = reduce_scatter([ranks[r].f2_attn_partial(q[r]) for r in R])
    tot = all_reduce([ranks[r].f3_moments(o[r]) for r in R])
    u = reduce_scatter([ranks[r].f4_up_partial(tot[r]) for r in R])
    d = reduce_scatter([ranks[r].f5_down_partial(u[r]) for r in R])
    y2 = [ranks[r].f6_finish(d[r]).clone() for r in R]
    full = all_gather([ranks[r].b0_start(dys[r]) for r in R])
    full = all_gather([ranks[r].b1_down(full[r]) for r in R])
    tot = all_reduce([ranks[r].b2_up(full[r]) for r in R])
    full = all_gather([ranks[r].b3_ln2(tot[r]) for r in R])
    full = all_gather([ranks[r].b4_attn(full[r]) for r in R])
    tot = all_reduce([ranks[r].b5_qkv(full[r]) for r in R])
    dx = [ranks[r].b6_ln1(tot[r]) for r in R]
    torch.cuda.synchronize()
    H2N = lambda t: t.float().cpu().numpy()   # noqa: E731
    return [H2N(t) for t in y2], [H2N(t) for t in dx], [{k: H2N(v) for k, v in ranks[r].grads.items()} for r in R]


@pytest.mark.parametrize("dtype,H,nh,I,T,S,Bz,causal", [
    ("f32", 256, 4, 512, 2, 128, 2, True),
    ("bf16", 1024, 16, 2048, 4, 256, 2, False),
    ("bf16", 512, 8, 1024, 2, 200, 1, True),
])
def test_simulated_ranks_match_oracle(dtype, H, nh, I, T, S, Bz, causal):
    import torch
    import paper_2111_05972_amd as pkg
    dt, eps = _dt(pkg, dtype), 1e-5
    print(f"\n[memopt-layer] {dtype} H={H} nh={nh} I={I} T={T} S={S} B={Bz} causal={causal}", flush=True)
    g = _global_params(1400, H, nh, I, dtype)
    M = S * Bz
    x = _draw(1450, (M, H), 1.0, dtype)
    dy = _draw(1451, (M, H), 1.0, dtype)
    shards = [mo.shard_reference_params(g, T, r) for r in range(T)]
    y2, dx, grads = _run_simulated_ranks(pkg, torch, dt, H, nh, I, T, S, Bz, causal, eps, shards, x, dy)
    Hs, nl, dh = H // T, nh // T, H // nh
    sl = lambda a: [a[:, r * Hs:(r + 1) * Hs] for r in range(T)]   # noqa: E731
    y_ref, sv = mo.memopt_layer_fwd(sl(x), shards, Bz, S, nl, dh, causal, eps)
    dx_ref, gr_ref = mo.memopt_layer_bwd(sl(dy), shards, sv, Bz, S, nl, dh)
    # the simulated ranks of the oracle are themselves the unsharded layer
    full_ref = mo.reference_layer_fwd(x, g, Bz, S, causal, eps)
    np.testing.assert_allclose(np.concatenate(y_ref, axis=1), full_ref, atol=1e-9)
    tol = TOL[dtype]                         # the benchmark spec's bound, end to end over all the pieces
    errs = {}
    errs["y2"] = max_rel_err(np.concatenate(y2, axis=1), full_ref)
    errs["dx"] = max_rel_err(np.concatenate(dx, axis=1), np.concatenate(dx_ref, axis=1))
    for r in range(T):
        for k, v in gr_ref[r].items():
            errs[f"r{r}.{k}"] = max_rel_err(grads[r][k], v)
    print("[memopt-layer] max-normalised errors: " + " ".join(f"{k}={e:.1e}" for k, e in errs.items()), flush=True)
    bad = {k: e for k, e in errs.items() if not e <= tol}
    assert not bad, f"over tolerance {tol}: {bad}"
