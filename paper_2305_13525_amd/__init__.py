"""MI355X-native shard GEMMs of a 3D-tensor-parallel fully-connected layer (AxoNN-style).

The product is the C-ABI library `libaxo.so` (HIP kernels for gfx950, declared in
include/axo.h); this package is the thin binding the tests and the benchmark call.
"""
from .binding import (  # noqa: F401
    AXO_EPI_BIAS, AXO_EPI_BIAS_GELU_ERF, AXO_EPI_BIAS_GELU_TANH, AXO_EPI_NONE,
    AXO_OP_DGRAD, AXO_OP_FWD, AXO_OP_WGRAD, AXO_ROUTE_COVERED, AXO_ROUTE_GENERAL, AXO_ROUTE_INTERIOR_STRIPS,
    AXO_ROUTE_NONE, AXO_ROUTE_TILED, AxoError, Layer, LayerExt, Problem,
    axo_bias_grad, axo_bias_grad_static, axo_bias_grad_static_limit,
    axo_bias_grad_workspace_bytes, axo_bias_grad_ws, axo_fc_dgrad, axo_fc_route, axo_fc_dgrad_act, axo_fc_fwd, axo_fc_wgrad, axo_fc_wgrad_acc, axo_layer_step,
    axo_layer_step_ext, axo_layer_step_levels, axo_layer_step_ordered, axo_layer_step_workspace_bytes,
    axo_shard_dims, axo_status_string, axo_version, axo_workspace_bytes, library, library_path,
)
