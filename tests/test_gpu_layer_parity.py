"""GPU parity: tp_layer_fwd / tp_layer_bwd through the C ABI against the float64 oracle,
element by element on the same seeded inputs (all outputs, all gradients, and the saved
intermediates).  Tolerances are the benchmark spec's bounds: 1e-4 (float) and 2e-2 (bfloat16) of each
tensor's max magnitude."""
import numpy as np
import pytest

import oracle
import synthetic
from synthetic.configs import small_variant

from gpu_util import compare, gpu_outputs, oracle_outputs, shard_inputs

pytestmark = pytest.mark.gpu

C = synthetic.CONFIGS


def _run(cfg):
    print(f"\n[case] {cfg.name} dtype={cfg.dtype} H={cfg.hidden} nh={cfg.heads} dh={cfg.head_dim} "
          f"T={cfg.tp_degree} r={cfg.tp_rank} S={cfg.seq} B={cfg.micro_batch} causal={cfg.causal} "
          f"epi={cfg.row_epilogue}", flush=True)
    d, sh = shard_inputs(cfg)
    got = gpu_outputs(cfg, d, sh)
    ref = oracle_outputs(cfg, d, sh)
    errs = compare(cfg, got, ref)
    print("  max rel err:", {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    return errs


# small shapes: several tiles, ragged tails in M, N and K, both masks, both epilogue settings, both dtypes
SMALL = [
    small_variant(C[1], name="f32-ragged", hidden=192, heads=6, head_dim=32, intermediate=776 * 2 // 2,
                  tp_degree=2, tp_rank=1, seq=75, micro_batch=3, causal=True, row_epilogue=False),
    small_variant(C[1], name="f32-bidir", hidden=128, heads=2, head_dim=64, intermediate=512,
                  tp_degree=1, tp_rank=0, seq=130, micro_batch=1, causal=False, row_epilogue=True),
    small_variant(C[2], name="bf16-ragged-causal", hidden=520, heads=5, head_dim=104, intermediate=2064,
                  tp_degree=1, tp_rank=0, seq=300, micro_batch=2, causal=True, row_epilogue=True),
    small_variant(C[2], name="bf16-tiles-bidir", hidden=768, heads=12, head_dim=64, intermediate=3072,
                  tp_degree=2, tp_rank=1, seq=384, micro_batch=2, causal=False, row_epilogue=False),
    small_variant(C[2], name="bf16-dh128-causal", hidden=1024, heads=8, head_dim=128, intermediate=4096,
                  tp_degree=4, tp_rank=2, seq=200, micro_batch=3, causal=True, row_epilogue=True),
    small_variant(C[2], name="bf16-seq1", hidden=256, heads=4, head_dim=64, intermediate=1024,
                  tp_degree=2, tp_rank=0, seq=1, micro_batch=8, causal=True, row_epilogue=True),
]


@pytest.mark.parametrize("cfg", SMALL, ids=[c.name for c in SMALL])
def test_small_shapes(cfg):
    _run(cfg)


@pytest.mark.parametrize("cid", [1, 2, 3])
def test_named_configs_small(cid):
    _run(C[cid])


@pytest.mark.parametrize("cid", [4, 5])
def test_named_configs_full_size(cid):
    """The GPT-3-shaped shards at full size, compared element by element (the oracle takes ~1 min)."""
    _run(C[cid])


@pytest.mark.parametrize("cid", [2, 3, 4, 5])
def test_two_chain_schedule_at_full_size(cid):
    """The launch configuration bench.py times: the attention block and the MLP block of a pass on two streams
    (TPL_SIDE_STREAM).  Element by element against the oracle, and bit-identical to the one-stream schedule (the
    kernels and their order within a chain are the same; only what runs beside what changes)."""
    cfg = C[cid]
    print(f"\n[case] two chains, {cfg.name}", flush=True)
    d, sh = shard_inputs(cfg)
    two = gpu_outputs(cfg, d, sh, side_stream=True)
    compare(cfg, two, oracle_outputs(cfg, d, sh))
    one = gpu_outputs(cfg, d, sh)
    for k in one:
        assert np.array_equal(one[k], two[k]), k


def test_three_chain_backward(tune):
    """Option side_chains = 3: dW_dn and dW_o, which depend on nothing computed in the pass, on a stream of their own.
    Against the oracle and bit-identical to the one-stream schedule."""
    tune.set("side_chains", "3")
    cfg = C[3]
    d, sh = shard_inputs(cfg)
    three = gpu_outputs(cfg, d, sh, side_stream=True)
    compare(cfg, three, oracle_outputs(cfg, d, sh))
    one = gpu_outputs(cfg, d, sh)
    for k in one:
        assert np.array_equal(one[k], three[k]), k


@pytest.mark.parametrize("name", sorted(synthetic.NEXT_SHAPES))
def test_paper_10b_encoder_shards(name):
    _run(synthetic.NEXT_SHAPES[name])


def test_flag_on_variant_of_headline_shape_small_seq():
    """Config 5's widths with the bias+residual epilogue on (shorter sequence keeps the oracle quick)."""
    _run(small_variant(C[5], name="gpt3-175b-tp8-epi", seq=256, row_epilogue=True))


@pytest.mark.parametrize("chunk", ["1", "2"])
def test_attention_strips_cut_into_chunks(chunk, tune):
    """The layer with its attention strips cut into chunks of 1 or 2 tile steps (partials in the workspace,
    combined by a second kernel), and the same twice over: bit-identical."""
    tune.set("attn_chunk", chunk)
    cfg = small_variant(C[2], name="bf16-dh128-causal-chunks", hidden=1024, heads=8, head_dim=128,
                        intermediate=2048, tp_degree=4, tp_rank=2, seq=333, micro_batch=2, causal=True,
                        row_epilogue=True)
    _run(cfg)
    d, sh = shard_inputs(cfg)
    a, b = gpu_outputs(cfg, d, sh, repeat=2)
    for k in a:
        assert np.array_equal(a[k], b[k]), k


@pytest.mark.parametrize("fuse", ["1", "0"])
def test_bias_gradients_inside_the_weight_gradient_gemm(fuse, tune):
    """db_qkv and db_up as one more output row of the weight-gradient GEMM (the 192 x 192 kernel forced for every
    GEMM so that small ragged shapes take that path: N = 1560 and 2064 are no multiples of the tile, the token count
    600 is no multiple of the k-step), and the same layer with the column-sum kernels instead; both against the
    oracle, and the fused result twice over bit-identical."""
    tune.set("gemm_tile", "7")
    tune.set("fuse_colsum", fuse)
    cfg = small_variant(C[2], name="bf16-colsum-in-wgrad", hidden=520, heads=5, head_dim=104, intermediate=2064,
                        tp_degree=1, tp_rank=0, seq=300, micro_batch=2, causal=True, row_epilogue=True)
    _run(cfg)
    d, sh = shard_inputs(cfg)
    a, b = gpu_outputs(cfg, d, sh, repeat=2)
    for k in ("db_qkv", "db_up"):
        assert np.array_equal(a[k], b[k]), k


def test_bias_gradients_inside_the_weight_gradient_gemm_at_full_size(tune):
    """The same option at config 5 with the library's own plans (its weight gradients run on the kernel that can carry
    the column sums): every tensor against the oracle."""
    tune.set("fuse_colsum", "1")
    _run(C[5])


def test_run_to_run_determinism():
    cfg = SMALL[3]
    d, sh = shard_inputs(cfg)
    a, b = gpu_outputs(cfg, d, sh, repeat=2)
    for k in a:
        assert np.array_equal(a[k], b[k]), k


def test_partials_of_all_ranks_sum_to_unsharded_layer_on_gpu():
    """Run every rank's shard on the one GPU; the sum of the partial outputs must be the unsharded
    layer (Fig. 7 caption; App. F.1), here checked against the oracle's unsharded layer."""
    cfg0 = small_variant(C[3], name="ranksum", hidden=512, heads=8, intermediate=2048, tp_degree=4,
                         seq=160, micro_batch=2, causal=True)
    d = synthetic.make_inputs(cfg0)
    ya_f, ym_f, sv = oracle.full_layer_fwd(d["x_a"], d["x_m"], d, cfg0.micro_batch, cfg0.seq, True)
    gr_f = oracle.full_layer_bwd(d["x_a"], d["x_m"], d, d["dy_a"], d["dy_m"], sv, cfg0.micro_batch, cfg0.seq, True)
    acc = {k: 0.0 for k in ("y_a", "y_m", "dx_a", "dx_m")}
    for r in range(cfg0.tp_degree):
        cfg = small_variant(cfg0, tp_rank=r, row_epilogue=(r == 0))
        got = gpu_outputs(cfg, d)            # sharded by the product's own rule
        for k in acc:
            acc[k] = acc[k] + got[k].astype(np.float64)
    ref = {"y_a": ya_f, "y_m": ym_f, "dx_a": gr_f["dx_a"], "dx_m": gr_f["dx_m"]}
    for k in acc:
        assert oracle.max_rel_err(acc[k], ref[k]) <= 2e-2, k
