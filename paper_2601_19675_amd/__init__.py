"""MI355X-native layer-wise post-training quantization solve (libptq bindings)."""
from .binding import (  # noqa: F401
    PTQ_BF16, PTQ_F32, PTQ_F64, PtqError, lib_path, load_library,
    ptq_activation_abs_sum, ptq_activation_scale, ptq_average_bits, ptq_damped_cholesky_inv, ptq_hessian_accumulate, ptq_layer_error,
    ptq_lopro_column_order, ptq_lopro_linear_forward, ptq_lopro_linear_forward_static, ptq_lopro_linear_forward_static_limit, ptq_lopro_rotate_hessian, ptq_lopro_rotate_weight, ptq_lopro_unrotate_weight,
    ptq_pack_codes, ptq_quantize_layer, ptq_quantize_layer_static_groups, ptq_quantize_layer_vq, ptq_scaled_r1svd, ptq_unpack_dequantize, ptq_status_string, ptq_workspace_bytes,
)
