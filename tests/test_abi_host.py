"""Host-side behaviour of the C ABI that needs no GPU: the library loads, exports every symbol the
header declares, validates descriptors, sizes buffers, and rejects bad calls before any launch."""
import ctypes
import os
import re

import pytest

import paper_2111_05972_amd as pkg
import synthetic

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib = pkg.load_library()
    text = open(os.path.join(ROOT, "include", "tp_layer.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(tp_layer_[a-z_]+)\s*\(", text))
    assert {"tp_layer_fwd", "tp_layer_bwd", "tp_layer_validate", "tp_layer_gemm"} <= names
    for n in names:
        assert hasattr(lib, n), n
    # the binding exposes the same names
    for n in names:
        assert hasattr(pkg, n), n


def test_struct_sizes_match_header():
    assert ctypes.sizeof(pkg.TpLayerDesc) == 40
    assert ctypes.sizeof(pkg.TpLayerParams) == 64 and ctypes.sizeof(pkg.TpLayerGrads) == 64
    assert ctypes.sizeof(pkg.TpLayerSavedLayout) == 48


def _desc(cfg, **kw):
    a = dict(hidden=cfg.hidden, heads=cfg.heads, tp_degree=cfg.tp_degree, tp_rank=cfg.tp_rank, seq=cfg.seq,
             micro_batch=cfg.micro_batch, dtype=pkg.TPL_F32 if cfg.dtype == "f32" else pkg.TPL_BF16,
             causal=cfg.causal, row_epilogue=cfg.row_epilogue, head_dim=cfg.head_dim, intermediate=cfg.intermediate)
    a.update(kw)
    return pkg.make_desc(**a)


@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5])
def test_named_configs_validate_and_size(cid):
    cfg = synthetic.CONFIGS[cid]
    d = _desc(cfg)
    assert pkg.tp_layer_validate(d) == pkg.TPL_OK
    es = 4 if cfg.dtype == "f32" else 2
    M, Hl, Il = cfg.tokens, cfg.local_attn, cfg.local_mlp
    need = M * 3 * Hl * es + M * Hl * es + cfg.micro_batch * cfg.local_heads * cfg.seq * 4 + 2 * M * Il * es
    got = pkg.tp_layer_saved_bytes(d)
    assert need <= got <= need + 5 * 256
    L = pkg.tp_layer_saved_offsets(d)
    assert L.qkv == 0 and L.qkv < L.o < L.lse < L.u < L.g < L.total == got
    assert all(o % 256 == 0 for o in (L.o, L.lse, L.u, L.g))
    assert pkg.tp_layer_workspace_bytes(d, 0) > 0
    assert pkg.tp_layer_workspace_bytes(d, 1) >= M * (Il + 4 * Hl) * es
    # head_dim / intermediate defaults
    d0 = _desc(cfg, head_dim=0, intermediate=0)
    assert pkg.tp_layer_saved_bytes(d0) == got


def test_invalid_descriptors():
    cfg = synthetic.CONFIGS[2]
    bad = [dict(heads=15), dict(tp_degree=3), dict(tp_rank=4), dict(tp_rank=-1), dict(seq=0), dict(micro_batch=-2),
           dict(hidden=0), dict(dtype=7), dict(head_dim=32), dict(intermediate=4098)]
    for kw in bad:
        d = _desc(cfg, **kw)
        assert pkg.tp_layer_validate(d) == pkg.TPL_EINVAL, kw
        assert pkg.tp_layer_saved_bytes(d) == 0 and pkg.tp_layer_workspace_bytes(d, 1) == 0
    d = _desc(cfg)
    d.flags = 8
    assert pkg.tp_layer_validate(d) == pkg.TPL_EINVAL
    d.flags = pkg.TPL_CAUSAL | pkg.TPL_SIDE_STREAM          # scheduling flag: a valid descriptor
    assert pkg.tp_layer_validate(d) == pkg.TPL_OK
    assert pkg.tp_layer_validate(None) == pkg.TPL_EINVAL
    # valid layers without a kernel
    assert pkg.tp_layer_validate(_desc(cfg, hidden=1020, heads=4, head_dim=255, intermediate=4080)) == pkg.TPL_EUNSUPPORTED
    assert pkg.tp_layer_validate(_desc(cfg, hidden=2048, heads=4, head_dim=512)) == pkg.TPL_EUNSUPPORTED


def test_calls_are_rejected_before_any_launch():
    """Null pointers, misalignment and short workspaces are caught on the host (runs without a GPU)."""
    cfg = synthetic.CONFIGS[2]
    d = _desc(cfg)
    ok = 0x1000     # never dereferenced: every call below fails validation first
    P = {k: ok for k in ("w_qkv", "b_qkv", "w_o", "b_o", "w_up", "b_up", "w_dn", "b_dn")}
    G = {"d" + k: ok for k in P}
    big = 1 << 40
    f = lambda **kw: pkg.tp_layer_fwd(d, kw.pop("params", P), kw.pop("x_attn", ok), ok, ok, ok, ok, ok,  # noqa: E731
                                      ws_bytes=kw.pop("ws_bytes", big), check=False)
    assert f(x_attn=None) == pkg.TPL_EINVAL
    assert f(params={**P, "w_up": None}) == pkg.TPL_EINVAL
    assert f(x_attn=ok + 8) == pkg.TPL_EALIGN
    assert f(ws_bytes=8) == pkg.TPL_EWORKSPACE
    d_epi = _desc(cfg, row_epilogue=True)
    assert pkg.tp_layer_fwd(d_epi, {**P, "b_o": None}, ok, ok, ok, ok, ok, ok, ws_bytes=big, check=False) == pkg.TPL_EINVAL
    b = lambda **kw: pkg.tp_layer_bwd(d, P, ok, ok, kw.pop("dy", ok), ok, ok, kw.pop("grads", G), ok, ok, ok,  # noqa: E731
                                      ws_bytes=kw.pop("ws_bytes", big), check=False)
    assert b(dy=None) == pkg.TPL_EINVAL
    assert b(grads={**G, "dw_dn": None}) == pkg.TPL_EINVAL
    assert b(grads={**G, "dw_o": ok + 2}) == pkg.TPL_EALIGN
    assert b(ws_bytes=pkg.tp_layer_workspace_bytes(d, 1) - 1) == pkg.TPL_EWORKSPACE
    with pytest.raises(pkg.TpLayerError):
        pkg.tp_layer_fwd(d, P, None, ok, ok, ok, ok, ok, ws_bytes=big)
    g = lambda **kw: pkg.tp_layer_gemm(kw.pop("dt", pkg.TPL_BF16), 0, 0, kw.pop("M", 64), 64, 64, kw.pop("A", ok), ok, ok,  # noqa: E731
                                       ws=ok, ws_bytes=big, check=False, **kw)
    assert g(A=None) == pkg.TPL_EINVAL and g(M=0) == pkg.TPL_EINVAL and g(dt=5) == pkg.TPL_EINVAL
    assert g(M=60) == pkg.TPL_EUNSUPPORTED and g(epi=pkg.TPL_EPI_GELU) == pkg.TPL_EINVAL
    assert pkg.tp_layer_attn_fwd(pkg.TPL_BF16, 1, 0, 1, 64, 1, ok, ok, ok, check=False) == pkg.TPL_EINVAL
    assert pkg.tp_layer_attn_fwd(pkg.TPL_BF16, 1, 8, 1, 512, 1, ok, ok, ok, check=False) == pkg.TPL_EUNSUPPORTED
    assert pkg.tp_layer_attn_bwd(pkg.TPL_F32, 1, 8, 1, 64, 1, ok, ok, ok, None, ok, ok, check=False) == pkg.TPL_EINVAL
    assert "workspace" in pkg.tp_layer_strerror(pkg.TPL_EWORKSPACE)


def test_forward_workspace_check_covers_the_attention_partials(tune):
    """With a forced attention chunk length the forward pass keeps float partials behind the two GEMM scratch
    halves: the size check of tp_layer_fwd is the size tp_layer_workspace_bytes reports, not the GEMM part alone."""
    cfg = synthetic.CONFIGS[4]
    d = _desc(cfg)
    ok, big = 0x1000, 1 << 40
    P = {k: ok for k in ("w_qkv", "b_qkv", "w_o", "b_o", "w_up", "b_up", "w_dn", "b_dn")}
    plain = pkg.tp_layer_workspace_bytes(d, 0)
    tune.set("attn_chunk", "2")
    forced = pkg.tp_layer_workspace_bytes(d, 0)
    assert forced > plain                                    # the partials of the cut strips
    f = lambda n: pkg.tp_layer_fwd(d, P, ok, ok, ok, ok, ok, ok, ws_bytes=n, check=False)   # noqa: E731
    assert f(plain) == pkg.TPL_EWORKSPACE                    # a buffer of the old size would be overrun
    assert f(forced - 1) == pkg.TPL_EWORKSPACE


def test_recompute_backward_validates_everything_before_enqueueing():
    """tp_layer_bwd_recompute runs a forward first: every argument of the backward part is checked before it."""
    cfg = synthetic.CONFIGS[3]                               # row epilogue on
    d = _desc(cfg)
    ok, big = 0x1000, 1 << 40
    P = {k: ok for k in ("w_qkv", "b_qkv", "w_o", "b_o", "w_up", "b_up", "w_dn", "b_dn")}
    G = {"d" + k: ok for k in P}

    def r(params=P, dy=ok, grads=G, dx=ok, ws=ok, ws_bytes=big):
        return pkg.tp_layer_bwd_recompute(d, params, ok, ok, dy, ok, grads, dx, ok, ws, ws_bytes=ws_bytes, check=False)
    assert r(dy=None) == pkg.TPL_EINVAL
    assert r(dx=None) == pkg.TPL_EINVAL
    assert r(grads={**G, "dw_qkv": None}) == pkg.TPL_EINVAL
    assert r(grads={**G, "db_o": None}) == pkg.TPL_EINVAL    # written on the epilogue rank
    assert r(grads={**G, "db_up": ok + 4}) == pkg.TPL_EALIGN
    assert r(dy=ok + 8) == pkg.TPL_EALIGN
    assert r(params={**P, "b_up": None}) == pkg.TPL_EINVAL   # the recomputed forward needs it
    assert r(ws_bytes=pkg.tp_layer_workspace_bytes_recompute(d) - 1) == pkg.TPL_EWORKSPACE


def test_options_are_set_through_the_abi_not_the_environment(tune, monkeypatch):
    ws = lambda: pkg.tp_layer_gemm_workspace_bytes(pkg.TPL_BF16, 512, 512, 4096)   # noqa: E731
    base = ws()
    monkeypatch.setenv("TPL_GEMM_SHARES", "3")               # the environment is read once, at load: no effect now
    assert ws() == base
    tune.set("gemm_shares", "3")
    assert ws() >= 3 * 512 * 512 * 4
    tune.set("gemm_shares", None)
    assert ws() == base
    assert pkg.tp_layer_set_option("no_such_option", "1", check=False) == pkg.TPL_EINVAL
    assert pkg.tp_layer_set_option("gemm_tile", "x", check=False) == pkg.TPL_EINVAL


def test_attention_workspace_follows_the_chunk_length(tune):
    """Partials of the cut strips: causal S = 300 has query strips of 2, 4, 5 tile steps and key strips of 5, 3, 1;
    with chunks of 2 steps that is 1 + 2 + 3 slots on the query side and 3 + 2 + 1 on the key side."""
    import paper_2111_05972_amd as pkg
    B, S, nl, dh = 2, 300, 3, 128
    tune.set("attn_chunk", "2")
    up = lambda n: (n + 255) // 256 * 256      # noqa: E731
    assert pkg.tp_layer_attn_workspace_bytes(pkg.TPL_BF16, B, S, nl, dh, 1, 0) == up(6 * B * nl * 128 * (dh + 2) * 4)
    assert pkg.tp_layer_attn_workspace_bytes(pkg.TPL_BF16, B, S, nl, dh, 1, 1) == up(6 * B * nl * 128 * 3 * dh * 4)
    assert pkg.tp_layer_attn_workspace_bytes(pkg.TPL_F32, B, S, nl, dh, 1, 0) == 0
    ok = 4096
    assert pkg.tp_layer_attn_fwd(pkg.TPL_BF16, B, S, nl, dh, 1, ok, ok, ok, ws=ok, ws_bytes=1024,
                                 check=False) == pkg.TPL_EWORKSPACE
    assert pkg.tp_layer_attn_bwd(pkg.TPL_BF16, B, S, nl, dh, 1, ok, ok, ok, ok, ok, ok, ws=ok, ws_bytes=1024,
                                 check=False) == pkg.TPL_EWORKSPACE
    tune.set("attn_chunk", "0")
    assert pkg.tp_layer_attn_workspace_bytes(pkg.TPL_BF16, B, S, nl, dh, 1, 1) == 0


def test_package_sharding_helper_matches_oracle_rule():
    import numpy as np
    import oracle
    d = synthetic.make_inputs(1)
    for r in range(2):
        a, b = pkg.shard_params(d, 2, r), oracle.shard_params(d, 2, r)
        for k in b:
            assert np.array_equal(np.asarray(a[k]), b[k]), k


def test_gemm_workspace_follows_the_k_share_plan(tune):
    """Host-side planning only: a GEMM with few tiles and a long K asks for float partial sums of whole shares,
    a GEMM that fills the chip asks for the minimum, and a forced share count is honoured."""
    tune.set("gemm_tile", None)
    tune.set("gemm_shares", None)
    ws = lambda M, N, K: pkg.tp_layer_gemm_workspace_bytes(pkg.TPL_BF16, M, N, K)   # noqa: E731
    few = ws(2048, 1536, 12288)                      # 64 tiles of 256 x 192 on 256 compute units
    assert few % (2048 * 1536 * 4) == 0 and 2 <= few // (2048 * 1536 * 4) <= 16
    assert ws(2048, 12288, 6144) == 256              # fills the chip: no split, minimum size
    assert ws(2048, 1536, 1024) == 256               # K too short to share
    tune.set("gemm_shares", "3")
    assert ws(512, 512, 4096) >= 3 * 512 * 512 * 4
    # the layer's workspace covers the split GEMMs of both chains of a pass
    tune.set("gemm_shares", None)
    cfg = synthetic.get_config(5)
    d = pkg.make_desc(cfg.hidden, cfg.heads, cfg.tp_degree, cfg.tp_rank, cfg.seq, cfg.micro_batch, pkg.TPL_BF16,
                      cfg.causal, cfg.row_epilogue, cfg.head_dim, cfg.intermediate)
    assert pkg.tp_layer_workspace_bytes(d, 1) >= 2 * few
