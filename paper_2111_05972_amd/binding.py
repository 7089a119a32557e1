"""ctypes binding of libtp_layer.so: same names as the C ABI, argument marshalling only.

Device buffers are anything with a `.data_ptr()` (torch tensors) or plain integer addresses.
There is no fallback: if the shared library is missing, loading raises.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libtp_layer.so"

TPL_OK, TPL_EINVAL, TPL_EUNSUPPORTED, TPL_EWORKSPACE, TPL_EALIGN, TPL_EHIP = range(6)
TPL_F32, TPL_BF16 = 0, 1
TPL_CAUSAL, TPL_ROW_EPILOGUE, TPL_SIDE_STREAM = 1, 2, 4
TPL_EPI_NONE, TPL_EPI_GELU, TPL_EPI_DGELU = 0, 1, 2
TPL_ACT_NONE, TPL_ACT_GELU = 0, 1

_vp = ctypes.c_void_p


class TpLayerDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("hidden", "heads", "head_dim", "intermediate", "tp_degree", "tp_rank", "seq",
                 "micro_batch", "dtype")] + [("flags", ctypes.c_uint32)]


class TpLayerParams(ctypes.Structure):
    _fields_ = [(n, _vp) for n in ("w_qkv", "b_qkv", "w_o", "b_o", "w_up", "b_up", "w_dn", "b_dn")]


class TpLayerGrads(ctypes.Structure):
    _fields_ = [(n, _vp) for n in ("dw_qkv", "db_qkv", "dw_o", "db_o", "dw_up", "db_up", "dw_dn", "db_dn")]


class TpLayerSavedLayout(ctypes.Structure):
    _fields_ = [(n, ctypes.c_size_t) for n in ("qkv", "o", "lse", "u", "g", "total")]


class TpLayerError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__(f"{what}: {tp_layer_strerror(status)} (status {status})")


_lib = None


def library_path():
    """The in-tree library; TPL_LIBRARY may name another build of the same sources (tuning experiments)."""
    return os.environ.get("TPL_LIBRARY") or os.path.join(_HERE, _LIB_NAME)


def load_library():
    """Load the HIP library built in-tree (python -m paper_2111_05972_amd.build). No fallback."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_2111_05972_amd.build` "
                          "(or __graft_entry__.build()); there is no non-HIP fallback")
    lib = ctypes.CDLL(path)
    D, P, G = ctypes.POINTER(TpLayerDesc), ctypes.POINTER(TpLayerParams), ctypes.POINTER(TpLayerGrads)
    i64, sz, ci = ctypes.c_int64, ctypes.c_size_t, ctypes.c_int
    sig = {
        "tp_layer_validate": (ci, [D]),
        "tp_layer_saved_bytes": (sz, [D]),
        "tp_layer_saved_offsets": (ci, [D, ctypes.POINTER(TpLayerSavedLayout)]),
        "tp_layer_workspace_bytes": (sz, [D, ci]),
        "tp_layer_fwd": (ci, [D, P, _vp, _vp, _vp, _vp, _vp, _vp, sz, _vp]),
        "tp_layer_bwd": (ci, [D, P, _vp, _vp, _vp, _vp, _vp, G, _vp, _vp, _vp, sz, _vp]),
        "tp_layer_gemm_workspace_bytes": (sz, [ci, i64, i64, i64]),
        "tp_layer_gemm": (ci, [ci, ci, ci, i64, i64, i64, _vp, _vp, _vp, _vp, _vp, _vp, ci, _vp, sz, _vp]),
        "tp_layer_attn_workspace_bytes": (sz, [ci, ci, ci, ci, ci, ci, ci]),
        "tp_layer_attn_fwd": (ci, [ci, ci, ci, ci, ci, ci, _vp, _vp, _vp, _vp, sz, _vp]),
        "tp_layer_attn_bwd": (ci, [ci, ci, ci, ci, ci, ci, _vp, _vp, _vp, _vp, _vp, _vp, _vp, sz, _vp]),
        "tp_layer_workspace_bytes_recompute": (sz, [D]),
        "tp_layer_bwd_recompute": (ci, [D, P, _vp, _vp, _vp, _vp, G, _vp, _vp, _vp, sz, _vp]),
        "tp_layer_ln_workspace_bytes": (sz, [i64, i64]),
        "tp_layer_ln_fwd": (ci, [ci, i64, i64, _vp, _vp, _vp, _vp, ctypes.c_float, _vp, _vp, _vp, _vp, _vp]),
        "tp_layer_ln_bwd": (ci, [ci, i64, i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, sz, _vp]),
        "tp_layer_ln_moments": (ci, [ci, i64, i64, _vp, _vp, _vp]),
        "tp_layer_ln_stats": (ci, [i64, i64, ctypes.c_float, _vp, _vp, _vp, _vp]),
        "tp_layer_ln_apply_fwd": (ci, [ci, i64, i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
        "tp_layer_ln_apply_bwd_sums": (ci, [ci, i64, i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
        "tp_layer_ln_apply_workspace_bytes": (sz, [i64, i64]),
        "tp_layer_ln_apply_bwd": (ci, [ci, i64, i64, i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, sz, _vp]),
        "tp_layer_slice_epilogue_fwd": (ci, [ci, ci, i64, i64, _vp, _vp, _vp, _vp, _vp, _vp]),
        "tp_layer_slice_epilogue_workspace_bytes": (sz, [i64, i64]),
        "tp_layer_slice_epilogue_bwd": (ci, [ci, ci, i64, i64, _vp, _vp, _vp, _vp, _vp, sz, _vp]),
        "tp_layer_static_scratch_bytes": (sz, []),
        "tp_layer_slice_epilogue_bwd_static": (ci, [ci, ci, i64, i64, _vp, _vp, _vp, _vp, _vp]),
        "tp_layer_set_option": (ci, [ctypes.c_char_p, ctypes.c_char_p]),
        "tp_layer_profile": (ci, [ci]),
        "tp_layer_profile_read": (ci, [ctypes.POINTER(ctypes.c_float), ci, ctypes.POINTER(ci)]),
        "tp_layer_strerror": (ctypes.c_char_p, [ci]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


def _ptr(x):
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    return int(x)


def _nbytes(x):
    return x.numel() * x.element_size() if hasattr(x, "numel") else None


def _stream(stream):
    if stream is None:
        return None
    return getattr(stream, "cuda_stream", stream)


def make_desc(hidden, heads, tp_degree, tp_rank, seq, micro_batch, dtype, causal, row_epilogue,
              head_dim=0, intermediate=0, side_stream=False):
    flags = ((TPL_CAUSAL if causal else 0) | (TPL_ROW_EPILOGUE if row_epilogue else 0) |
             (TPL_SIDE_STREAM if side_stream else 0))
    return TpLayerDesc(hidden, heads, head_dim, intermediate, tp_degree, tp_rank, seq, micro_batch,
                       dtype, flags)


def _params(p):
    if isinstance(p, TpLayerParams):
        return p
    return TpLayerParams(*[_ptr(p.get(n)) for n, _ in TpLayerParams._fields_])


def _grads(g):
    if isinstance(g, TpLayerGrads):
        return g
    return TpLayerGrads(*[_ptr(g.get(n)) for n, _ in TpLayerGrads._fields_])


def tp_layer_strerror(status):
    return load_library().tp_layer_strerror(int(status)).decode()


def tp_layer_validate(desc):
    return load_library().tp_layer_validate(ctypes.byref(desc) if desc is not None else None)


def tp_layer_saved_bytes(desc):
    return load_library().tp_layer_saved_bytes(ctypes.byref(desc))


def tp_layer_saved_offsets(desc):
    out = TpLayerSavedLayout()
    rc = load_library().tp_layer_saved_offsets(ctypes.byref(desc), ctypes.byref(out))
    if rc != TPL_OK:
        raise TpLayerError(rc, "tp_layer_saved_offsets")
    return out


def tp_layer_workspace_bytes(desc, bwd):
    return load_library().tp_layer_workspace_bytes(ctypes.byref(desc), int(bool(bwd)))


def tp_layer_fwd(desc, params, x_attn, x_mlp, y_attn_partial, y_mlp_partial, saved, ws,
                 ws_bytes=None, stream=None, check=True):
    pr = _params(params)
    rc = load_library().tp_layer_fwd(
        ctypes.byref(desc), ctypes.byref(pr), _ptr(x_attn), _ptr(x_mlp), _ptr(y_attn_partial),
        _ptr(y_mlp_partial), _ptr(saved), _ptr(ws), _nbytes(ws) if ws_bytes is None else ws_bytes,
        _stream(stream))
    if check and rc != TPL_OK:
        raise TpLayerError(rc, "tp_layer_fwd")
    return rc


def tp_layer_bwd(desc, params, x_attn, x_mlp, dy_attn, dy_mlp, saved, grads, dx_attn_partial,
                 dx_mlp_partial, ws, ws_bytes=None, stream=None, check=True):
    pr, gr = _params(params), _grads(grads)
    rc = load_library().tp_layer_bwd(
        ctypes.byref(desc), ctypes.byref(pr), _ptr(x_attn), _ptr(x_mlp), _ptr(dy_attn), _ptr(dy_mlp),
        _ptr(saved), ctypes.byref(gr), _ptr(dx_attn_partial), _ptr(dx_mlp_partial), _ptr(ws),
        _nbytes(ws) if ws_bytes is None else ws_bytes, _stream(stream))
    if check and rc != TPL_OK:
        raise TpLayerError(rc, "tp_layer_bwd")
    return rc


def tp_layer_workspace_bytes_recompute(desc):
    return load_library().tp_layer_workspace_bytes_recompute(ctypes.byref(desc))


def tp_layer_bwd_recompute(desc, params, x_attn, x_mlp, dy_attn, dy_mlp, grads, dx_attn_partial,
                           dx_mlp_partial, ws, ws_bytes=None, stream=None, check=True):
    pr, gr = _params(params), _grads(grads)
    rc = load_library().tp_layer_bwd_recompute(
        ctypes.byref(desc), ctypes.byref(pr), _ptr(x_attn), _ptr(x_mlp), _ptr(dy_attn), _ptr(dy_mlp),
        ctypes.byref(gr), _ptr(dx_attn_partial), _ptr(dx_mlp_partial), _ptr(ws),
        _nbytes(ws) if ws_bytes is None else ws_bytes, _stream(stream))
    if check and rc != TPL_OK:
        raise TpLayerError(rc, "tp_layer_bwd_recompute")
    return rc


def tp_layer_ln_workspace_bytes(M, H):
    return load_library().tp_layer_ln_workspace_bytes(M, H)


def tp_layer_ln_fwd(dtype, M, H, a, b, gamma, beta, eps, z, y, mean, rstd, stream=None, check=True):
    rc = load_library().tp_layer_ln_fwd(dtype, M, H, _ptr(a), _ptr(b), _ptr(gamma), _ptr(beta), float(eps),
                                        _ptr(z), _ptr(y), _ptr(mean), _ptr(rstd), _stream(stream))
    if check and rc != TPL_OK:
        raise TpLayerError(rc, "tp_layer_ln_fwd")
    return rc


def tp_layer_ln_bwd(dtype, M, H, dy, z, mean, rstd, gamma, dz, dgamma, dbeta, ws, ws_bytes=None, stream=None,
                    check=True):
    rc = load_library().tp_layer_ln_bwd(dtype, M, H, _ptr(dy), _ptr(z), _ptr(mean), _ptr(rstd), _ptr(gamma),
                                        _ptr(dz), _ptr(dgamma), _ptr(dbeta), _ptr(ws),
                                        (_nbytes(ws) or 0) if ws_bytes is None else ws_bytes, _stream(stream))
    if check and rc != TPL_OK:
        raise TpLayerError(rc, "tp_layer_ln_bwd")
    return rc


def _checked(rc, what, check):
    if check and rc != TPL_OK:
        raise TpLayerError(rc, what)
    return rc


def tp_layer_ln_moments(dtype, M, Hs, x_loc, sums, stream=None, check=True):
    rc = load_library().tp_layer_ln_moments(dtype, M, Hs, _ptr(x_loc), _ptr(sums), _stream(stream))
    return _checked(rc, "tp_layer_ln_moments", check)


def tp_layer_ln_stats(M, H, eps, totals, mean, rstd, stream=None, check=True):
    rc = load_library().tp_layer_ln_stats(M, H, float(eps), _ptr(totals), _ptr(mean), _ptr(rstd), _stream(stream))
    return _checked(rc, "tp_layer_ln_stats", check)


def tp_layer_ln_apply_fwd(dtype, M, Hs, x_loc, mean, rstd, gamma_loc, beta_loc, y, stream=None, check=True):
    rc = load_library().tp_layer_ln_apply_fwd(dtype, M, Hs, _ptr(x_loc), _ptr(mean), _ptr(rstd), _ptr(gamma_loc),
                                              _ptr(beta_loc), _ptr(y), _stream(stream))
    return _checked(rc, "tp_layer_ln_apply_fwd", check)


def tp_layer_ln_apply_bwd_sums(dtype, M, Hs, dy, x_loc, mean, rstd, gamma_loc, sums, stream=None, check=True):
    rc = load_library().tp_layer_ln_apply_bwd_sums(dtype, M, Hs, _ptr(dy), _ptr(x_loc), _ptr(mean), _ptr(rstd),
                                                   _ptr(gamma_loc), _ptr(sums), _stream(stream))
    return _checked(rc, "tp_layer_ln_apply_bwd_sums", check)


def tp_layer_ln_apply_workspace_bytes(M, Hs):
    return load_library().tp_layer_ln_apply_workspace_bytes(M, Hs)


def tp_layer_ln_apply_bwd(dtype, M, Hs, H, dy, x_loc, mean, rstd, gamma_loc, totals, dx_add, dx, dgamma_loc,
                          dbeta_loc, ws, ws_bytes=None, stream=None, check=True):
    rc = load_library().tp_layer_ln_apply_bwd(
        dtype, M, Hs, H, _ptr(dy), _ptr(x_loc), _ptr(mean), _ptr(rstd), _ptr(gamma_loc), _ptr(totals), _ptr(dx_add),
        _ptr(dx), _ptr(dgamma_loc), _ptr(dbeta_loc), _ptr(ws), (_nbytes(ws) or 0) if ws_bytes is None else ws_bytes,
        _stream(stream))
    return _checked(rc, "tp_layer_ln_apply_bwd", check)


def tp_layer_slice_epilogue_fwd(dtype, act, M, N, inp, bias, resid, u, out, stream=None, check=True):
    rc = load_library().tp_layer_slice_epilogue_fwd(dtype, act, M, N, _ptr(inp), _ptr(bias), _ptr(resid), _ptr(u),
                                                    _ptr(out), _stream(stream))
    return _checked(rc, "tp_layer_slice_epilogue_fwd", check)


def tp_layer_slice_epilogue_workspace_bytes(M, N):
    return load_library().tp_layer_slice_epilogue_workspace_bytes(M, N)


def tp_layer_slice_epilogue_bwd(dtype, act, M, N, dout, u, din, dbias, ws, ws_bytes=None, stream=None, check=True):
    rc = load_library().tp_layer_slice_epilogue_bwd(dtype, act, M, N, _ptr(dout), _ptr(u), _ptr(din), _ptr(dbias),
                                                    _ptr(ws), (_nbytes(ws) or 0) if ws_bytes is None else ws_bytes,
                                                    _stream(stream))
    return _checked(rc, "tp_layer_slice_epilogue_bwd", check)


def tp_layer_static_scratch_bytes():
    return load_library().tp_layer_static_scratch_bytes()


def tp_layer_slice_epilogue_bwd_static(dtype, act, M, N, dout, u, din, dbias, stream=None, check=True):
    rc = load_library().tp_layer_slice_epilogue_bwd_static(dtype, act, M, N, _ptr(dout), _ptr(u), _ptr(din),
                                                           _ptr(dbias), _stream(stream))
    return _checked(rc, "tp_layer_slice_epilogue_bwd_static", check)


def tp_layer_set_option(name, value=None, check=True):
    """Tuning override (see tp_layer.h); value None or "" returns the option to the library's own choice."""
    v = None if value is None else str(value).encode()
    rc = load_library().tp_layer_set_option(name.encode(), v)
    return _checked(rc, f"tp_layer_set_option({name})", check)


def tp_layer_profile(enable):
    return load_library().tp_layer_profile(int(bool(enable)))


def tp_layer_profile_read(capacity=4096):
    """Durations (ms) of the GEMM launches recorded since profiling was enabled, in launch order."""
    buf = (ctypes.c_float * capacity)()
    n = ctypes.c_int(0)
    rc = load_library().tp_layer_profile_read(buf, capacity, ctypes.byref(n))
    if rc != TPL_OK:
        raise TpLayerError(rc, "tp_layer_profile_read")
    return [buf[i] for i in range(n.value)]


def tp_layer_gemm_workspace_bytes(dtype, M, N, K):
    return load_library().tp_layer_gemm_workspace_bytes(dtype, M, N, K)


def tp_layer_gemm(dtype, trans_a, trans_b, M, N, K, A, B, C, bias=None, resid=None, aux=None,
                  epi=TPL_EPI_NONE, ws=None, ws_bytes=None, stream=None, check=True):
    rc = load_library().tp_layer_gemm(
        dtype, int(bool(trans_a)), int(bool(trans_b)), M, N, K, _ptr(A), _ptr(B), _ptr(C), _ptr(bias),
        _ptr(resid), _ptr(aux), epi, _ptr(ws), (_nbytes(ws) or 0) if ws_bytes is None else ws_bytes,
        _stream(stream))
    if check and rc != TPL_OK:
        raise TpLayerError(rc, "tp_layer_gemm")
    return rc


def tp_layer_attn_workspace_bytes(dtype, B, S, nl, dh, causal, bwd):
    return load_library().tp_layer_attn_workspace_bytes(dtype, B, S, nl, dh, int(bool(causal)), int(bool(bwd)))


def tp_layer_attn_fwd(dtype, B, S, nl, dh, causal, qkv, o, lse, ws=None, ws_bytes=None, stream=None,
                      check=True):
    rc = load_library().tp_layer_attn_fwd(dtype, B, S, nl, dh, int(bool(causal)), _ptr(qkv), _ptr(o),
                                          _ptr(lse), _ptr(ws),
                                          (_nbytes(ws) or 0) if ws_bytes is None else ws_bytes, _stream(stream))
    if check and rc != TPL_OK:
        raise TpLayerError(rc, "tp_layer_attn_fwd")
    return rc


def tp_layer_attn_bwd(dtype, B, S, nl, dh, causal, qkv, o, lse, d_o, dqkv, d_scratch, ws=None,
                      ws_bytes=None, stream=None, check=True):
    rc = load_library().tp_layer_attn_bwd(dtype, B, S, nl, dh, int(bool(causal)), _ptr(qkv), _ptr(o),
                                          _ptr(lse), _ptr(d_o), _ptr(dqkv), _ptr(d_scratch), _ptr(ws),
                                          (_nbytes(ws) or 0) if ws_bytes is None else ws_bytes, _stream(stream))
    if check and rc != TPL_OK:
        raise TpLayerError(rc, "tp_layer_attn_bwd")
    return rc
