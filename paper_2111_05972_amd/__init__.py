"""MI355X-native forward/backward of one tensor-parallel rank's transformer-layer shard.

The computation lives in hand-written HIP kernels behind the C ABI declared in
include/tp_layer.h; this package only loads that library and marshals arguments.
"""
from .binding import (  # noqa: F401
    TPL_OK, TPL_EINVAL, TPL_EUNSUPPORTED, TPL_EWORKSPACE, TPL_EALIGN, TPL_EHIP,
    TPL_F32, TPL_BF16, TPL_CAUSAL, TPL_ROW_EPILOGUE, TPL_SIDE_STREAM, TPL_EPI_NONE, TPL_EPI_GELU, TPL_EPI_DGELU,
    TpLayerDesc, TpLayerParams, TpLayerGrads, TpLayerSavedLayout, TpLayerError,
    library_path, load_library, make_desc,
    tp_layer_validate, tp_layer_saved_bytes, tp_layer_saved_offsets, tp_layer_workspace_bytes,
    tp_layer_fwd, tp_layer_bwd, tp_layer_gemm, tp_layer_gemm_workspace_bytes,
    tp_layer_attn_workspace_bytes, tp_layer_attn_fwd, tp_layer_attn_bwd, tp_layer_strerror, tp_layer_profile, tp_layer_profile_read, tp_layer_set_option,
    tp_layer_workspace_bytes_recompute, tp_layer_bwd_recompute,
    tp_layer_ln_workspace_bytes, tp_layer_ln_fwd, tp_layer_ln_bwd,
    tp_layer_ln_moments, tp_layer_ln_stats, tp_layer_ln_apply_fwd, tp_layer_ln_apply_bwd_sums,
    tp_layer_ln_apply_workspace_bytes, tp_layer_ln_apply_bwd,
    tp_layer_slice_epilogue_fwd, tp_layer_slice_epilogue_workspace_bytes, tp_layer_slice_epilogue_bwd,
    TPL_ACT_NONE, TPL_ACT_GELU, tp_layer_static_scratch_bytes, tp_layer_slice_epilogue_bwd_static,
)


def __getattr__(name):
    # torch-backed helpers are imported on first use so that the ABI can be loaded without torch
    if name in ("TpLayer", "shard_params", "to_device", "PARAM_NAMES", "GRAD_NAMES"):
        from . import layer
        return getattr(layer, name)
    raise AttributeError(name)
