"""The seeded input generator: determinism, distribution, bf16 storage rounding."""
import numpy as np
import torch

import synthetic
from synthetic import gen


def test_chunking_and_seed_independence():
    a = gen.normal(123, 1000, 2.0)
    b = gen.normal(123, 1000, 2.0, chunk=37)
    assert np.array_equal(a, b)
    assert not np.array_equal(a, gen.normal(124, 1000, 2.0))


def test_moments():
    x = gen.normal(5, 1 << 20, 0.02).astype(np.float64)
    assert abs(x.mean()) < 1e-4 and abs(x.std() - 0.02) < 1e-4
    z = x / 0.02
    assert abs((z ** 3).mean()) < 0.02 and abs((z ** 4).mean() - 3.0) < 0.05


def test_bf16_rounding_matches_torch():
    x = gen.normal(9, 1 << 16, 1.0)
    x[:4] = [1.00390625, 1.01171875, -1.00390625, 0.0]     # ties: to even
    bits = gen.to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(bits.view(np.int16), ref.view(torch.int16).numpy())
    assert np.array_equal(gen.bf16_bits_to_f32(bits), ref.float().numpy())
    q = gen.quantize(x, "bf16")
    assert np.array_equal(gen.quantize(q, "bf16"), q)


def test_configs_shapes_and_flops():
    c = synthetic.CONFIGS[5]
    assert (c.tokens, c.local_heads, c.local_attn, c.local_mlp) == (2048, 12, 1536, 6144)
    f, b = c.flops()
    assert abs((f + b) / 1e12 - 2.822) < 2e-3
    tot = [sum(synthetic.CONFIGS[i].flops()) / 1e12 for i in range(1, 6)]
    assert np.allclose(tot, [0.00063, 0.0838, 0.335, 1.997, 2.822], rtol=2e-2)
    d = synthetic.make_inputs(1)
    assert d["Wqkv"].shape == (256, 3, 4, 64) and d["x_a"].shape == (256, 256)
    assert abs(d["x_a"].std() - 0.02) < 1e-3 and abs(d["dy_a"].std() - 1.0) < 2e-2
    d2 = synthetic.make_inputs(1, only=["Wo"])
    assert np.array_equal(d2["Wo"], d["Wo"])
