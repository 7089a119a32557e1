"""CPU oracle for the tensor-parallel transformer-layer shard.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package.  It shares no code with the GPU path and never imports it.
"""
from .tp_layer_oracle import (  # noqa: F401
    shard_params, layer_fwd, layer_bwd, full_layer_fwd, full_layer_bwd,
    gelu, gelu_grad, attention_fwd, attention_bwd, max_rel_err, layernorm_fwd, layernorm_bwd,
)
