"""Buffer management around the C ABI: allocate device memory with torch, call the library.

No arithmetic happens here; every step of the path runs in the HIP kernels.
"""
import numpy as np
import torch

from . import binding as B

_TORCH_DTYPE = {B.TPL_F32: torch.float32, B.TPL_BF16: torch.bfloat16}
PARAM_NAMES = ("w_qkv", "b_qkv", "w_o", "b_o", "w_up", "b_up", "w_dn", "b_dn")
GRAD_NAMES = ("dw_qkv", "db_qkv", "dw_o", "db_o", "dw_up", "db_up", "dw_dn", "db_dn")


def shard_params(g, T, r):
    """Rank r's slices of unsharded parameters (pure indexing; works on numpy arrays and tensors).

    First linears are split over output channels (heads / MLP columns), second linears over input
    channels (rows); row-parallel biases are passed whole and used only by the epilogue rank.
    """
    H, three, nh, dh = g["Wqkv"].shape
    nl, Il = nh // T, g["Wup"].shape[1] // T
    return {
        "w_qkv": g["Wqkv"][:, :, r * nl:(r + 1) * nl, :].reshape(H, 3 * nl * dh),
        "b_qkv": g["bqkv"][:, r * nl:(r + 1) * nl, :].reshape(3 * nl * dh),
        "w_o": g["Wo"][r * nl * dh:(r + 1) * nl * dh, :],
        "b_o": g["bo"],
        "w_up": g["Wup"][:, r * Il:(r + 1) * Il],
        "b_up": g["bup"][r * Il:(r + 1) * Il],
        "w_dn": g["Wdn"][r * Il:(r + 1) * Il, :],
        "b_dn": g["bdn"],
    }


def to_device(x, dtype, device="cuda"):
    """Host array holding dtype-representable float32 values -> contiguous device tensor."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    return t.to(device=device, dtype=_TORCH_DTYPE[dtype]).contiguous()


class TpLayer:
    """One rank's layer shard: owns saved/workspace buffers and calls tp_layer_fwd / tp_layer_bwd."""

    def __init__(self, hidden, heads, tp_degree, tp_rank, seq, micro_batch, dtype, causal,
                 row_epilogue, head_dim=0, intermediate=0, device="cuda", side_stream=False):
        self.desc = B.make_desc(hidden, heads, tp_degree, tp_rank, seq, micro_batch, dtype, causal,
                                row_epilogue, head_dim, intermediate, side_stream)
        rc = B.tp_layer_validate(self.desc)
        if rc != B.TPL_OK:
            raise B.TpLayerError(rc, "tp_layer_validate")
        self.dtype = dtype
        self.tdtype = _TORCH_DTYPE[dtype]
        self.device = device
        self.H = hidden
        self.dh = head_dim or hidden // heads
        self.nl = heads // tp_degree
        self.Hl = self.nl * self.dh
        self.Il = (intermediate or 4 * hidden) // tp_degree
        self.M = seq * micro_batch
        self.B, self.S = micro_batch, seq
        self.saved = torch.empty(B.tp_layer_saved_bytes(self.desc), dtype=torch.uint8, device=device)
        nws = max(B.tp_layer_workspace_bytes(self.desc, 0), B.tp_layer_workspace_bytes(self.desc, 1))
        self.ws = torch.empty(nws, dtype=torch.uint8, device=device)
        self.layout = B.tp_layer_saved_offsets(self.desc)

    def param_shapes(self):
        H, Hl, Il = self.H, self.Hl, self.Il
        return {"w_qkv": (H, 3 * Hl), "b_qkv": (3 * Hl,), "w_o": (Hl, H), "b_o": (H,),
                "w_up": (H, Il), "b_up": (Il,), "w_dn": (Il, H), "b_dn": (H,)}

    def empty_outputs(self):
        mk = lambda: torch.empty(self.M, self.H, dtype=self.tdtype, device=self.device)  # noqa: E731
        return mk(), mk()

    def empty_grads(self):
        return {"d" + k: torch.empty(s, dtype=self.tdtype, device=self.device)
                for k, s in self.param_shapes().items()}

    def forward(self, params, x_attn, x_mlp, y_attn=None, y_mlp=None, stream=None):
        if y_attn is None:
            y_attn, y_mlp = self.empty_outputs()
        st = stream if stream is not None else torch.cuda.current_stream()
        B.tp_layer_fwd(self.desc, params, x_attn, x_mlp, y_attn, y_mlp, self.saved, self.ws, stream=st)
        return y_attn, y_mlp

    def backward(self, params, x_attn, x_mlp, dy_attn, dy_mlp, grads=None, dx_attn=None, dx_mlp=None,
                 stream=None):
        if grads is None:
            grads = self.empty_grads()
        if dx_attn is None:
            dx_attn, dx_mlp = self.empty_outputs()
        st = stream if stream is not None else torch.cuda.current_stream()
        B.tp_layer_bwd(self.desc, params, x_attn, x_mlp, dy_attn, dy_mlp, self.saved, grads, dx_attn,
                       dx_mlp, self.ws, stream=st)
        return grads, dx_attn, dx_mlp

    def saved_tensors(self):
        """Views of what forward kept: QKV, O, LSE, U, G."""
        L, M = self.layout, self.M
        es = 4 if self.dtype == B.TPL_F32 else 2

        def view(off, shape, dt, esz):
            n = int(np.prod(shape))
            return self.saved[off:off + n * esz].view(dt).reshape(shape)
        return {
            "QKV": view(L.qkv, (M, 3 * self.Hl), self.tdtype, es),
            "O": view(L.o, (M, self.Hl), self.tdtype, es),
            "LSE": view(L.lse, (self.B, self.nl, self.S), torch.float32, 4),
            "U": view(L.u, (M, self.Il), self.tdtype, es),
            "G": view(L.g, (M, self.Il), self.tdtype, es),
        }
