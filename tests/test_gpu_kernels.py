"""Per-kernel GPU parity through the C ABI: every GEMM transpose/epilogue combination and the
attention forward/backward, against the oracle's definitions."""
import numpy as np
import pytest

import oracle
import synthetic

pytestmark = pytest.mark.gpu


def _t(x, dt):
    import paper_2111_05972_amd as pkg
    return pkg.to_device(x, dt)


def _draw(seed, shape, sigma, dtype):
    n = int(np.prod(shape))
    return synthetic.quantize(synthetic.normal(seed, n, sigma), dtype).reshape(shape)


GEMM_SHAPES = [(256, 256, 64), (520, 264, 136), (1000, 776, 2056), (64, 1536, 4096), (8, 8, 8), (264, 512, 72),
               (2048, 1536, 3080), (4104, 4360, 520)]


# bf16 runs once per tile variant of the MFMA kernel (forced through the option gemm_tile) and once with the
# library's own choice; float has a single kernel.
def _check_gemms(dtype, tile, shares, ta, tb, epi, shapes, tune):
    import torch
    import paper_2111_05972_amd as pkg
    for name, val in (("gemm_tile", tile), ("gemm_shares", shares)):
        tune.set(name, val)
    dt = pkg.TPL_BF16 if dtype == "bf16" else pkg.TPL_F32
    tol = 2e-2 if dtype == "bf16" else 1e-4
    for si, (M, N, K) in enumerate(shapes):
        print(f"\n[gemm] {dtype} ta={ta} tb={tb} epi={epi} M={M} N={N} K={K}", flush=True)
        A = _draw(100 + si, (K, M) if ta else (M, K), 1.0, dtype)
        B = _draw(200 + si, (N, K) if tb else (K, N), 0.05, dtype)
        bias = _draw(300 + si, (N,), 0.5, dtype)
        resid = _draw(400 + si, (M, N), 1.0, dtype)
        aux_in = _draw(500 + si, (M, N), 1.0, dtype)
        A64 = (A.T if ta else A).astype(np.float64)
        B64 = (B.T if tb else B).astype(np.float64)
        ref = A64 @ B64
        ref_aux = None
        kw = {}
        if epi in ("bias", "bias_resid", "gelu"):
            ref = ref + bias
            kw["bias"] = _t(bias, dt)
        if epi == "bias_resid":
            ref = ref + resid
            kw["resid"] = _t(resid, dt)
        C = torch.empty(M, N, dtype=kw.get("bias", _t(bias, dt)).dtype, device="cuda")
        aux = None
        if epi == "gelu":
            ref_aux = ref
            ref = oracle.gelu(ref)
            aux = torch.empty_like(C)
            kw.update(aux=aux, epi=pkg.TPL_EPI_GELU)
        if epi == "dgelu":
            ref = ref * oracle.gelu_grad(aux_in)
            aux = _t(aux_in, dt)
            kw.update(aux=aux, epi=pkg.TPL_EPI_DGELU)
        ws = torch.empty(pkg.tp_layer_gemm_workspace_bytes(dt, M, N, K), dtype=torch.uint8, device="cuda")
        pkg.tp_layer_gemm(dt, ta, tb, M, N, K, _t(A, dt), _t(B, dt), C, ws=ws,
                          stream=torch.cuda.current_stream(), **kw)
        torch.cuda.synchronize()
        err = oracle.max_rel_err(C.float().cpu().numpy(), ref)
        assert err <= tol, (M, N, K, err)
        if ref_aux is not None:
            assert oracle.max_rel_err(aux.float().cpu().numpy(), ref_aux) <= tol


@pytest.mark.parametrize("dtype,tile", [("bf16", None), ("bf16", "0"), ("bf16", "1"), ("bf16", "2"), ("bf16", "3"), ("bf16", "4"), ("bf16", "5"), ("bf16", "6"), ("bf16", "7"), ("f32", None)])
@pytest.mark.parametrize("ta,tb", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("epi", ["none", "bias", "bias_resid", "gelu", "dgelu"])
def test_gemm_variants(dtype, tile, ta, tb, epi, tune):
    _check_gemms(dtype, tile, None, ta, tb, epi, GEMM_SHAPES, tune)


# K cut into shares (one workgroup per tile and share, partial sums added in share order by a second kernel):
# forced share counts on every tile variant, K not a multiple of the share length, a share count above the
# number of k-steps, and the library's own choice on a few-tiles / long-K shape where it splits by itself.
SPLIT_SHAPES = [(256, 192, 520), (520, 264, 1096), (264, 512, 72), (8, 8, 8), (1000, 776, 2056)]


@pytest.mark.parametrize("tile", [None, "0", "1", "2", "3", "4", "5", "6", "7"])
@pytest.mark.parametrize("shares", ["2", "5"])
@pytest.mark.parametrize("ta,tb", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("epi", ["bias_resid", "gelu", "dgelu"])
def test_gemm_k_shares(tile, shares, ta, tb, epi, tune):
    _check_gemms("bf16", tile, shares, ta, tb, epi, SPLIT_SHAPES, tune)


@pytest.mark.parametrize("ta,tb", [(0, 0), (0, 1), (1, 0)])
def test_gemm_k_shares_own_choice(ta, tb, tune):
    import paper_2111_05972_amd as pkg
    tune.set("gemm_tile", None)
    tune.set("gemm_shares", None)
    M, N, K = 512, 384, 8200
    assert pkg.tp_layer_gemm_workspace_bytes(pkg.TPL_BF16, M, N, K) >= 2 * M * N * 4     # it does split
    _check_gemms("bf16", None, None, ta, tb, "bias_resid", [(M, N, K)], tune)


ATTN_CASES = [(2, 128, 2, 64), (1, 300, 3, 128), (3, 77, 2, 32), (1, 1, 4, 64), (2, 513, 1, 64), (1, 1024, 2, 128)]


@pytest.mark.parametrize("causal", [True, False])
def test_attention_long_sequence_own_chunk_length(causal, tune):
    """S = 4096 on two heads: far fewer strips than compute units, so with a workspace the library cuts them by
    its own rule (several chunks per strip, also without a mask); forward and backward against the oracle."""
    import torch
    import paper_2111_05972_amd as pkg
    tune.set("attn_chunk", None)
    B, S, nl, dh, dt, tol = 1, 4096, 2, 128, pkg.TPL_BF16, 2e-2
    print(f"\n[attn] long S causal={causal} B={B} S={S} nl={nl} dh={dh}", flush=True)
    nf, nb = (pkg.tp_layer_attn_workspace_bytes(dt, B, S, nl, dh, causal, bwd) for bwd in (False, True))
    assert nf > 0 and nb > 0
    qkv = _draw(900, (B * S, 3 * nl * dh), 1.0, "bf16")
    d_o = _draw(901, (B * S, nl * dh), 1.0, "bf16")
    t = qkv.reshape(B, S, 3, nl, dh).astype(np.float64)
    Q, K, V = (t[:, :, i].transpose(0, 2, 1, 3) for i in range(3))
    O, P, LSE = oracle.attention_fwd(Q, K, V, causal)
    qkv_d = _t(qkv, dt)
    o_d = torch.empty(B * S, nl * dh, dtype=qkv_d.dtype, device="cuda")
    lse_d = torch.empty(B, nl, S, dtype=torch.float32, device="cuda")
    ws_f = torch.full((nf // 4,), float("nan"), dtype=torch.float32, device="cuda")
    ws_b = torch.full((nb // 4,), float("nan"), dtype=torch.float32, device="cuda")
    st = torch.cuda.current_stream()
    pkg.tp_layer_attn_fwd(dt, B, S, nl, dh, causal, qkv_d, o_d, lse_d, ws=ws_f, stream=st)
    torch.cuda.synchronize()
    assert oracle.max_rel_err(o_d.float().cpu().numpy(), O.transpose(0, 2, 1, 3).reshape(B * S, nl * dh)) <= tol
    assert np.abs(lse_d.cpu().numpy() - LSE).max() <= 2e-2
    dO = d_o.reshape(B, S, nl, dh).transpose(0, 2, 1, 3).astype(np.float64)
    dQ, dK, dV = oracle.attention_bwd(Q, K, V, P, dO)
    ref = np.stack([a.transpose(0, 2, 1, 3) for a in (dQ, dK, dV)], axis=2).reshape(B * S, 3 * nl * dh)
    dqkv_d = torch.empty_like(qkv_d)
    scratch = torch.empty(B, nl, S, dtype=torch.float32, device="cuda")
    pkg.tp_layer_attn_bwd(dt, B, S, nl, dh, causal, qkv_d, o_d, lse_d, _t(d_o, dt), dqkv_d, scratch, ws=ws_b, stream=st)
    torch.cuda.synchronize()
    got = dqkv_d.float().cpu().numpy()
    for i, nm in enumerate(("dQ", "dK", "dV")):
        sl = slice(i * nl * dh, (i + 1) * nl * dh)
        assert oracle.max_rel_err(got[:, sl], ref[:, sl]) <= tol, nm


# chunk: None = no workspace (strips never cut); "auto" = workspace, the library's own chunk length;
# "1", "3" = workspace and chunks of that many 64-row tile steps (every strip longer than that is cut).
@pytest.mark.parametrize("dtype,chunk", [("bf16", None), ("bf16", "auto"), ("bf16", "1"), ("bf16", "3"), ("f32", None)])
@pytest.mark.parametrize("causal", [True, False])
def test_attention_fwd_bwd(dtype, chunk, causal, tune):
    import torch
    import paper_2111_05972_amd as pkg
    dt = pkg.TPL_BF16 if dtype == "bf16" else pkg.TPL_F32
    tol = 2e-2 if dtype == "bf16" else 1e-4
    tune.set("attn_chunk", None)
    if chunk not in (None, "auto"):
        tune.set("attn_chunk", chunk)
    for ci, (B, S, nl, dh) in enumerate(ATTN_CASES):
        print(f"\n[attn] {dtype} causal={causal} chunk={chunk} B={B} S={S} nl={nl} dh={dh}", flush=True)
        ws_f = ws_b = None
        if chunk is not None:
            nf, nb = (pkg.tp_layer_attn_workspace_bytes(dt, B, S, nl, dh, causal, bwd) for bwd in (False, True))
            if chunk == "1" and S > 64 and dh in (64, 128):
                assert nf > 0 and nb > 0                       # these strips are cut
            # filled with NaN: a partial that is read without having been written shows up
            ws_f = torch.full((max(nf, 16) // 4,), float("nan"), dtype=torch.float32, device="cuda")
            ws_b = torch.full((max(nb, 16) // 4,), float("nan"), dtype=torch.float32, device="cuda")
        qkv = _draw(700 + ci, (B * S, 3 * nl * dh), 1.0, dtype)
        d_o = _draw(800 + ci, (B * S, nl * dh), 1.0, dtype)
        t = qkv.reshape(B, S, 3, nl, dh).astype(np.float64)
        Q, K, V = (t[:, :, i].transpose(0, 2, 1, 3) for i in range(3))
        O, P, LSE = oracle.attention_fwd(Q, K, V, causal)
        o_ref = O.transpose(0, 2, 1, 3).reshape(B * S, nl * dh)
        qkv_d = _t(qkv, dt)
        o_d = torch.empty(B * S, nl * dh, dtype=qkv_d.dtype, device="cuda")
        lse_d = torch.empty(B, nl, S, dtype=torch.float32, device="cuda")
        st = torch.cuda.current_stream()
        pkg.tp_layer_attn_fwd(dt, B, S, nl, dh, causal, qkv_d, o_d, lse_d, ws=ws_f, stream=st)
        torch.cuda.synchronize()
        assert oracle.max_rel_err(o_d.float().cpu().numpy(), o_ref) <= tol
        assert np.abs(lse_d.cpu().numpy() - LSE).max() <= (2e-2 if dtype == "bf16" else 1e-4)
        # backward takes the O the forward stored (as the layer does)
        dO = d_o.reshape(B, S, nl, dh).transpose(0, 2, 1, 3).astype(np.float64)
        dQ, dK, dV = oracle.attention_bwd(Q, K, V, P, dO)
        ref = np.stack([a.transpose(0, 2, 1, 3) for a in (dQ, dK, dV)], axis=2).reshape(B * S, 3 * nl * dh)
        dqkv_d = torch.empty_like(qkv_d)
        scratch = torch.empty(B, nl, S, dtype=torch.float32, device="cuda")
        pkg.tp_layer_attn_bwd(dt, B, S, nl, dh, causal, qkv_d, o_d, lse_d, _t(d_o, dt), dqkv_d, scratch, ws=ws_b,
                              stream=st)
        torch.cuda.synchronize()
        got = dqkv_d.float().cpu().numpy()
        for i, nm in enumerate(("dQ", "dK", "dV")):
            sl = slice(i * nl * dh, (i + 1) * nl * dh)
            assert oracle.max_rel_err(got[:, sl], ref[:, sl]) <= tol, (nm, B, S, nl, dh)
