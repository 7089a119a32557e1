"""Named workload shapes and their seeded tensors.

Shapes follow the tensor-parallel layer description (hidden size H, nh heads of
size dh, MLP width I, tensor-parallel degree T, rank r, sequence S, micro-batch
B).  Each tensor has its own seed so any of them can be regenerated alone.
"""
from dataclasses import dataclass, replace
import numpy as np

from .gen import normal, quantize

BASE_SEED = 211105972
TENSOR_IDS = {name: i for i, name in enumerate(
    ["x_a", "x_m", "Wqkv", "bqkv", "Wo", "bo", "Wup", "bup", "Wdn", "bdn", "dy_a", "dy_m"])}


@dataclass(frozen=True)
class LayerConfig:
    name: str
    cfg_id: int
    dtype: str            # 'f32' or 'bf16' (storage type of every tensor the GPU path sees)
    hidden: int
    heads: int
    head_dim: int
    intermediate: int
    tp_degree: int
    tp_rank: int
    seq: int
    micro_batch: int
    causal: bool
    row_epilogue: bool    # this rank adds the row-parallel biases and the residual
    sigma_w: float = 0.02
    sigma_x: float = 1.0
    sigma_dy: float = 1.0
    global_params: bool = True   # generate unsharded parameters (else the shard directly)

    @property
    def tokens(self):
        return self.seq * self.micro_batch

    @property
    def local_heads(self):
        return self.heads // self.tp_degree

    @property
    def local_attn(self):
        return self.local_heads * self.head_dim

    @property
    def local_mlp(self):
        return self.intermediate // self.tp_degree

    def flops(self):
        """Model flops (fwd, bwd): GEMMs 2MNK (bwd 2x); attention 4*B*nl*pairs*dh (bwd 2x)."""
        M, H, Hl, Il = self.tokens, self.hidden, self.local_attn, self.local_mlp
        gemm = 2.0 * M * H * (3 * Hl + Hl + Il + Il)
        pairs = self.seq * (self.seq + 1) / 2 if self.causal else float(self.seq) ** 2
        attn = 4.0 * self.micro_batch * self.local_heads * pairs * self.head_dim
        fwd = gemm + attn
        return fwd, 2.0 * fwd


CONFIGS = {
    1: LayerConfig("tiny-gpt-f32", 1, "f32", 256, 4, 64, 1024, 2, 0, 128, 2, True, True,
                   sigma_w=0.02, sigma_x=0.02, sigma_dy=1.0),
    2: LayerConfig("bert-large-tp4", 2, "bf16", 1024, 16, 64, 4096, 4, 1, 512, 8, False, False),
    3: LayerConfig("roberta-large-tp2", 3, "bf16", 1024, 16, 64, 4096, 2, 0, 512, 16, False, True),
    4: LayerConfig("gpt3-13b-tp4", 4, "bf16", 5120, 40, 128, 20480, 4, 0, 2048, 2, True, True,
                   global_params=False),
    5: LayerConfig("gpt3-175b-tp8", 5, "bf16", 12288, 96, 128, 49152, 8, 3, 2048, 1, True, False,
                   sigma_w=0.006, global_params=False),
}

# The 10B encoder shards the paper trained (Table 1), as extra shapes.
NEXT_SHAPES = {
    "roberta-10b-tp4": LayerConfig("roberta-10b-tp4", 6, "bf16", 4096, 32, 128, 16384, 4, 0, 512, 8,
                                   False, True, global_params=False),
    "bert-10b-tp4": LayerConfig("bert-10b-tp4", 7, "bf16", 2560, 40, 64, 10240, 4, 0, 512, 8,
                                False, True, global_params=False),
}


def get_config(key):
    if isinstance(key, LayerConfig):
        return key
    if key in CONFIGS:
        return CONFIGS[key]
    if key in NEXT_SHAPES:
        return NEXT_SHAPES[key]
    raise KeyError(key)


def small_variant(cfg, **kw):
    """Same recipe at another size (for tests)."""
    return replace(cfg, **kw)


def _draw(cfg, name, shape, sigma):
    n = int(np.prod(shape))
    seed = BASE_SEED + 1000 * cfg.cfg_id + TENSOR_IDS[name]
    return quantize(normal(seed, n, sigma), cfg.dtype).reshape(shape)


def make_inputs(cfg, only=None):
    """Seeded tensors of a config as float32 arrays holding `cfg.dtype`-representable values.

    Activations x_a, x_m and upstream gradients dy_a, dy_m are [tokens, hidden].
    With cfg.global_params the parameters are the unsharded ones
    (Wqkv [H,3,nh,dh], bqkv [3,nh,dh], Wo [nh*dh,H], bo [H], Wup [H,I], bup [I], Wdn [I,H], bdn [H]);
    otherwise they have the shapes of one rank's shard
    (Wqkv [H,3,nl,dh], bqkv [3,nl,dh], Wo [nl*dh,H], Wup [H,Il], bup [Il], Wdn [Il,H]).
    """
    cfg = get_config(cfg)
    M, H = cfg.tokens, cfg.hidden
    if cfg.global_params:
        nh, I = cfg.heads, cfg.intermediate
    else:
        nh, I = cfg.local_heads, cfg.local_mlp
    dh = cfg.head_dim
    shapes = {
        "x_a": ((M, H), cfg.sigma_x), "x_m": ((M, H), cfg.sigma_x),
        "Wqkv": ((H, 3, nh, dh), cfg.sigma_w), "bqkv": ((3, nh, dh), cfg.sigma_w),
        "Wo": ((nh * dh, H), cfg.sigma_w), "bo": ((H,), cfg.sigma_w),
        "Wup": ((H, I), cfg.sigma_w), "bup": ((I,), cfg.sigma_w),
        "Wdn": ((I, H), cfg.sigma_w), "bdn": ((H,), cfg.sigma_w),
        "dy_a": ((M, H), cfg.sigma_dy), "dy_m": ((M, H), cfg.sigma_dy),
    }
    names = list(shapes) if only is None else list(only)
    return {k: _draw(cfg, k, *shapes[k]) for k in names}
