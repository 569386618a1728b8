"""libmesa: Mesa's activation-compression hot path (arXiv 2111.11124) as HIP kernels for MI355X.

The product is the C-ABI shared library declared in include/mesa.h; this package is its thin
Python binding (same names, argument marshalling only).
"""
from ._ffi import (  # noqa: F401
    F16, F32, BF16, ROUND_NEAREST_EVEN, ROUND_STOCHASTIC,
    OP_UPDATE_RUNNING_PARAMS, OP_LAYERNORM_BWD_Q, OP_LINEAR_DW_Q, OP_SOFTMAX_FWD_Q, OP_LAYERNORM_FWD_Q,
    OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_LAUNCH,
    EXPORTS, Conv2d, Event, Layout, MesaError, lib, status_string, version, workspace_bytes,
    mesa_update_running_params, mesa_update_running_params_sym, mesa_update_running_params_fixed_beta, mesa_update_running_scale_sym, mesa_quantize_sym, mesa_dequantize_sym, mesa_update_running_params_static, static_scratch_bytes, mesa_quantize_headwise, mesa_quantize_update_fused, mesa_gelu_fwd_q, mesa_softmax_fwd_q, mesa_layernorm_fwd_q, mesa_dequantize, mesa_quantize_headwise_b4, mesa_dequantize_b4, mesa_gelu_bwd_q_b4, mesa_softmax_bwd_q,
    mesa_gelu_bwd_q, mesa_relu_bwd_q, mesa_layernorm_bwd_q, mesa_linear_dw_q, mesa_conv2d_dw_q, conv2d_dw_q_workspace_bytes, mesa_attn_av_bwd_q, mesa_attn_qk_bwd_q, mesa_stream_copy, mesa_stream_read, mesa_stream_fill, mesa_mfma_probe, MFMA_PROBE_WAVES, MFMA_PROBE_FLOPS_PER_STEP,
)
