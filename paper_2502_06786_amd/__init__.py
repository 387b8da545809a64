"""MI355X-native nested quantized linear layer of Matryoshka Quantization (arXiv 2502.06786).

The implementation is the HIP library ``libmq.so`` (C ABI in ``include/mq.h``); ``binding`` marshals
torch tensors into it.  The binding is loaded on first use and raises ImportError when the library
has not been built: there is no other implementation to fall back to.
"""
_BINDING_NAMES = {
    "mq_quantize_int8", "mq_slice", "mq_linear_fwd_multi", "mq_linear_bwd", "mq_gemv_sliced", "mq_params_to_bf16",
    "mq_workspace_bytes", "mq_gemv_sliced_dense_ep", "MQ_FLAG_EP_DENSE", "status_string", "Overflow", "MqError", "lib", "LIB_PATH", "EXPORTS",
    "MQ_FLAG_EXTRA_PRECISION", "MQ_FLAG_PACKED", "MQ_FLAG_ACCUM_DW", "MQ_OP_LINEAR_FWD", "MQ_OP_LINEAR_BWD",
    "mq_ffn_mixnmatch", "MQ_OP_FFN_DECODE", "MQ_FLAG_FFN_SILU", "MQ_FLAG_FFN_RESIDUAL",
    "mq_matquant_l2_loss", "MQ_OP_L2_LOSS", "MQ_FLAG_LOSS_MIX", "mq_linear_fwd_multi_l2", "MQ_OP_LINEAR_FWD_L2", "mq_linear_bwd_clip", "MQ_OP_LINEAR_BWD_CLIP", "mq_affine_weight", "mq_affine_input", "mq_affine_bwd", "MQ_OP_AFFINE_BWD", "mq_gated_unit_fwd", "mq_gated_unit_bwd", "mq_linear_fwd_multi_noalloc", "mq_linear_bwd_gated", "mq_slice_multi", "mq_linear_fwd_multi_gated", "mq_gemv_sliced_ws", "MQ_OP_GEMV",
}


def __getattr__(name):
    if name in _BINDING_NAMES:
        from . import binding
        return getattr(binding, name)
    raise AttributeError(name)
